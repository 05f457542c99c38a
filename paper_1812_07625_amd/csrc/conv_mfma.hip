// Temporal convolution as implicit GEMM on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16: bf16 operands, fp32 accumulation).
//
// The three passes of the convolution the paper's network is built from (Sec. 2.3,
// Sec. 4.1) are each one GEMM D[m,n] = sum_r A[m,r] * B[n,r] whose operands are read
// straight from the channels-last tensors -- the time window of a frame is a contiguous
// run of k*C elements, so no unfolded copy exists anywhere:
//
//   fwd    m=(b,t')  n=co      r=(j,ci)   A = x window (r-contiguous)   B = w[co] (r-contiguous)
//   dgrad  m=(b,t)   n=ci      r=(j',co)  A = dy window (r-contiguous)  B = w (n-contiguous), j'=k-1-j
//   wgrad  m=co      n=(j,ci)  r=(b,t')   A = dy (m-contiguous)         B = x window (n-contiguous)
//
// One workgroup = 4 wavefronts (2x2) computes a BM x BN tile; each wavefront owns a
// (BM/2)x(BN/2) sub-tile of 32x32 MFMA blocks held in registers.  Operand panels of
// BK reduction steps are fetched global -> registers -> LDS (double buffered, one
// barrier per step).  r-contiguous panels are stored [row][BK] with a 16-byte row pad
// and read with one 16-byte LDS read per MFMA operand; m/n-contiguous panels are
// stored [BK][row] and read through the LDS transpose read (ds_read_b64_tr_b16), which
// hands each lane the 4 consecutive reduction elements of its row.  Zero padding at
// the utterance edges, ragged tiles and the reduction tail are all handled by
// predicating the 16-byte global loads; stores are predicated on the tile bounds.
#include "common.h"

namespace w2l {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int NT = 256;       // threads per workgroup
constexpr int BK = 64;        // reduction elements per panel
constexpr int KPAD = 16;      // bytes of padding per r-contiguous LDS row
constexpr int MNPAD = 64;     // bytes of padding per m/n-contiguous LDS row

struct ConvGeom {
    int B, T, Tp, Cin, Cout, k, s, p;
};

// ---- r-contiguous panel: ROWS rows x BK elements -------------------------------------
// Row i of the tile is a run of memory starting at element offset `off` (may point
// before the tensor for halo rows); reduction index r is valid in [lo, hi).
template <int ROWS>
struct PanelK {
    static constexpr int RS = BK * 2 + KPAD;            // LDS row stride in bytes
    static constexpr int BYTES = ROWS * RS;
    static constexpr int CPR = BK / 8;                  // 16-byte chunks per row
    static constexpr int NCH = ROWS * CPR / NT;         // chunks per thread
    static constexpr int READS_PER_FRAG = 1;
    static_assert(ROWS * CPR % NT == 0, "panel must divide over the workgroup");
    int off[NCH];                                      // element offsets (tensors hold < 2^31 elements)
    int lo[NCH], hi[NCH];
    uint4 reg[NCH];
    int c8;                                             // this thread's element offset inside a row
    const bf16_t* base;

    __device__ __forceinline__ int row_of(int i) const { return (threadIdx.x + i * NT) / CPR; }
    __device__ __forceinline__ void issue(int r0)
    {
        const int r = r0 + c8;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (r >= lo[i] && r < hi[i]) v = *reinterpret_cast<const uint4*>(base + off[i] + r);
            reg[i] = v;
        }
    }
    __device__ __forceinline__ void commit(unsigned char* lds) const
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            *reinterpret_cast<uint4*>(lds + row_of(i) * RS + c8 * 2) = reg[i];
    }
    // 32 rows starting at row0, reduction sub-step ks (16 elements): lane holds row l%32, r = 8*(l/32)..+7
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int row0, int ks, int lane)
    {
        const unsigned char* p = lds + (row0 + (lane & 31)) * RS + (ks * 16 + 8 * (lane >> 5)) * 2;
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const s16x8*>(p));
    }
};

// ---- m/n-contiguous panel: BK reduction rows x COLS elements ---------------------------
// Reduction row i (of this step) starts at element offset rowoff(i); columns valid in
// [lo, hi).  The caller supplies the per-step row addressing to issue().
template <int COLS>
struct PanelMN {
    static constexpr int RS = COLS * 2 + MNPAD;
    static constexpr int BYTES = BK * RS;
    static constexpr int CPR = COLS / 8;
    static constexpr int NCH = BK * CPR / NT;
    static constexpr int READS_PER_FRAG = 2;
    static_assert(BK * CPR % NT == 0, "panel must divide over the workgroup");
    uint4 reg[NCH];
    const bf16_t* base;

    __device__ __forceinline__ void init(const bf16_t* b) { base = b; }
    static __device__ __forceinline__ int row_of(int i) { return (threadIdx.x + i * NT) / CPR; }
    static __device__ __forceinline__ int col_of(int i) { return ((threadIdx.x + i * NT) % CPR) * 8; }
    // f(row, off, lo, hi): element offset of the row's column 0 of this tile and the valid
    // column range; the 16-byte chunk at column c is loaded iff lo <= c < hi
    template <class F>
    __device__ __forceinline__ void issue(F f)
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            long long off;
            int lo, hi;
            const int c8 = col_of(i);
            f(row_of(i), off, lo, hi);
            uint4 v = make_uint4(0, 0, 0, 0);
            if (c8 >= lo && c8 < hi) v = *reinterpret_cast<const uint4*>(base + off + c8);
            reg[i] = v;
        }
    }
    __device__ __forceinline__ void commit(unsigned char* lds) const
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            *reinterpret_cast<uint4*>(lds + row_of(i) * RS + col_of(i) * 2) = reg[i];
    }
    // same fragment as PanelK::frag, gathered with two transpose reads: within each group of
    // 16 lanes, lane i supplies the address of row (i/4), columns 4*(i%4)..+3 and receives
    // column i of rows 0..3
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int col0, int ks, int lane)
    {
        const int q = lane >> 4, i = lane & 15;
        const int col = col0 + 16 * (q & 1) + 4 * (i & 3);
        const int r = ks * 16 + 8 * (q >> 1) + (i >> 2);
        const unsigned char* p = lds + r * RS + col * 2;
        const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
        const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * RS));
        s16x8 v;
        v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
        v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
        return __builtin_bit_cast(bf16x8, v);
    }
};

// ---- the 2x2-wavefront MFMA core ----------------------------------------------------
template <int BM, int BN, class PA, class PB>
struct Core {
    static constexpr int TM = BM / 2 / 32, TN = BN / 2 / 32;  // 32x32 blocks per wavefront
    f32x16 acc[TM][TN];
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    }
    // One panel (BK reduction elements).  Operand fragments are double-buffered in
    // registers: the LDS reads of sub-step ks+1 are issued before the MFMAs of sub-step ks,
    // so their latency hides under matrix work (one wavefront per SIMD: nothing else would).
    __device__ __forceinline__ void step(const unsigned char* la, const unsigned char* lb, int wm, int wn, int lane)
    {
        constexpr int NS = BK / 16;
        bf16x8 a[2][TM], b[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[0][i] = PA::frag(la, wm * (BM / 2) + i * 32, 0, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[0][j] = PB::frag(lb, wn * (BN / 2) + j * 32, 0, lane);
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            const int c = ks & 1, n = c ^ 1;
            if (ks + 1 < NS) {
#pragma unroll
                for (int i = 0; i < TM; ++i) a[n][i] = PA::frag(la, wm * (BM / 2) + i * 32, ks + 1, lane);
#pragma unroll
                for (int j = 0; j < TN; ++j) b[n][j] = PB::frag(lb, wn * (BN / 2) + j * 32, ks + 1, lane);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // f(m, n, value) for every element this lane holds; m,n relative to the tile
    template <class F>
    __device__ __forceinline__ void for_each(int wm, int wn, int lane, F f) const
    {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const int n = wn * (BN / 2) + j * 32 + (lane & 31);
                    f(m, n, acc[i][j][r]);
                }
    }
};

// Workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its own
// L2); give each XCD a contiguous run of tiles, ordered with the shorter grid dimension
// fastest, so that the tiles sharing an L2 cover a compact block of operand panels.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn)
{
    const int nb = tiles_m * tiles_n;
    const int per = (nb + 7) / 8;
    int id = (blockIdx.x % 8) * per + blockIdx.x / 8;
    if (nb % 8 != 0) id = blockIdx.x;  // keep it a bijection when the count does not split evenly
    if (tiles_n <= tiles_m) { tm = id / tiles_n; tn = id % tiles_n; }
    else { tn = id / tiles_m; tm = id % tiles_m; }
}

// =============================== forward ================================================
template <int BM, int BN, typename TO>
__global__ __launch_bounds__(NT) void conv_fwd_k(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                 const float* __restrict__ bias, TO* __restrict__ y, ConvGeom g)
{
    using PA = PanelK<BM>;
    using PB = PanelK<BN>;
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int STAGE = PA::BYTES + PB::BYTES;  // stage i holds [A panel | B panel]
    const int M = g.B * g.Tp, N = g.Cout, K = g.k * g.Cin;
    int tm, tn;
    tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;

    PA pa;
    PB pb;
    pa.base = x;
    pb.base = w;
    pa.c8 = (threadIdx.x % PA::CPR) * 8;
    pb.c8 = pa.c8;
#pragma unroll
    for (int i = 0; i < PA::NCH; ++i) {
        const int m = m0 + pa.row_of(i);
        const int b = m / g.Tp, tp = m - b * g.Tp;
        const int t0 = g.s * tp - g.p;                  // first frame of the window (may be < 0)
        pa.off[i] = (b * g.T + t0) * g.Cin;
        pa.lo[i] = (t0 < 0 ? -t0 : 0) * g.Cin;
        const int last = g.T - t0;                      // taps j < last are inside the utterance
        pa.hi[i] = (m < M) ? (last < g.k ? last : g.k) * g.Cin : 0;
    }
#pragma unroll
    for (int i = 0; i < PB::NCH; ++i) {
        const int n = n0 + pb.row_of(i);
        pb.off[i] = n * K;
        pb.lo[i] = 0;
        pb.hi[i] = (n < N) ? K : 0;
    }
    Core<BM, BN, PA, PB> core;
    core.zero();
    const int nsteps = (K + BK - 1) / BK;
    pa.issue(0);
    pb.issue(0);
    pa.commit(lds);
    pb.commit(lds + PA::BYTES);
    __syncthreads();
    for (int st = 0; st < nsteps; ++st) {
        unsigned char* cur = lds + (st & 1) * STAGE;
        unsigned char* nxt = lds + ((st & 1) ^ 1) * STAGE;
        if (st + 1 < nsteps) { pa.issue((st + 1) * BK); pb.issue((st + 1) * BK); }
        core.step(cur, cur + PA::BYTES, wm, wn, lane);
        if (st + 1 < nsteps) { pa.commit(nxt); pb.commit(nxt + PA::BYTES); }
        __syncthreads();
    }
    core.for_each(wm, wn, lane, [&](int mm, int nn, float v) {
        const int m = m0 + mm, n = n0 + nn;
        if (m < M && n < N) Elem<TO>::store(y, (size_t)m * N + n, v + (bias ? bias[n] : 0.f));
    });
}

// =============================== data gradient (stride 1) =============================
// dx[b,t,ci] = sum_{j',co} dy[b, t-p+j', co] * w[co, k-1-j', ci]
template <int BM, int BN>
__global__ __launch_bounds__(NT) void conv_dgrad_k(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ w,
                                                   bf16_t* __restrict__ dx, ConvGeom g)
{
    using PA = PanelK<BM>;
    using PB = PanelMN<BN>;
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int STAGE = PA::BYTES + PB::BYTES;  // stage i holds [A panel | B panel]
    const int M = g.B * g.T, N = g.Cin, K = g.k * g.Cout;
    int tm, tn;
    tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;

    PA pa;
    PB pb;
    pa.base = dy;
    pa.c8 = (threadIdx.x % PA::CPR) * 8;
    pb.init(w);
#pragma unroll
    for (int i = 0; i < PA::NCH; ++i) {
        const int m = m0 + pa.row_of(i);
        const int b = m / g.T, t = m - b * g.T;
        const int t0 = t - g.p;
        pa.off[i] = (b * g.Tp + t0) * g.Cout;
        pa.lo[i] = (t0 < 0 ? -t0 : 0) * g.Cout;
        const int last = g.Tp - t0;
        pa.hi[i] = (m < M) ? (last < g.k ? last : g.k) * g.Cout : 0;
    }
    // reduction row r = (j', co): Cout is a multiple of BK, so a step stays inside one tap
    auto wrow = [&](int st) {
        const int r0 = st * BK;
        const int jp = r0 / g.Cout, co0 = r0 - jp * g.Cout;
        const long long tapoff = (long long)(g.k - 1 - jp) * g.Cin + n0;
        const int ncols = N - n0;
        return [=](int rr, long long& off, int& lo, int& hi) {
            off = (long long)(co0 + rr) * g.k * g.Cin + tapoff;
            lo = 0;
            hi = ncols;  // chunk columns are multiples of 8 and N % 8 == 0
        };
    };
    Core<BM, BN, PA, PB> core;
    core.zero();
    const int nsteps = K / BK;
    pa.issue(0);
    pb.issue(wrow(0));
    pa.commit(lds);
    pb.commit(lds + PA::BYTES);
    __syncthreads();
    for (int st = 0; st < nsteps; ++st) {
        unsigned char* cur = lds + (st & 1) * STAGE;
        unsigned char* nxt = lds + ((st & 1) ^ 1) * STAGE;
        if (st + 1 < nsteps) { pa.issue((st + 1) * BK); pb.issue(wrow(st + 1)); }
        core.step(cur, cur + PA::BYTES, wm, wn, lane);
        if (st + 1 < nsteps) { pa.commit(nxt); pb.commit(nxt + PA::BYTES); }
        __syncthreads();
    }
    core.for_each(wm, wn, lane, [&](int mm, int nn, float v) {
        const int m = m0 + mm, n = n0 + nn;
        if (m < M && n < N) dx[(size_t)m * N + n] = f32_to_bf16(v);
    });
}

// =============================== weight gradient ========================================
// dw[co, (j,ci)] = sum_{b,t'} dy[b,t',co] * x[b, s t' - p + j, ci]; the reduction walks
// utterance by utterance in BK-frame steps (the last step of an utterance is masked).
template <int BM, int BN>
__global__ __launch_bounds__(NT) void conv_wgrad_k(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                   float* __restrict__ dw, ConvGeom g, int accumulate)
{
    using PA = PanelMN<BM>;
    using PB = PanelMN<BN>;
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int STAGE = PA::BYTES + PB::BYTES;  // stage i holds [A panel | B panel]
    const int M = g.Cout, N = g.k * g.Cin;
    int tm, tn;
    tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;

    PA pa;
    PB pb;
    pa.init(dy);
    pb.init(x);
    const int spb = (g.Tp + BK - 1) / BK;  // steps per utterance
    const int nsteps = g.B * spb;
    auto arow = [&](int st) {
        const int b = st / spb, tp0 = (st - b * spb) * BK;
        const long long boff = ((long long)b * g.Tp + tp0) * g.Cout + m0;
        const int left = g.Tp - tp0, ncols = M - m0;
        return [=](int rr, long long& off, int& lo, int& hi) {
            off = boff + (long long)rr * g.Cout;
            lo = 0;
            hi = (rr < left) ? ncols : 0;
        };
    };
    auto brow = [&](int st) {
        const int b = st / spb, tp0 = (st - b * spb) * BK;
        const int left = g.Tp - tp0;
        return [=](int rr, long long& off, int& lo, int& hi) {
            const int t0 = g.s * (tp0 + rr) - g.p;               // frame under tap 0
            off = ((long long)b * g.T + t0) * g.Cin + n0;
            // tile column c <-> tap-major index n0 + c ; valid taps: 0 <= t0 + j < T
            const int jlo = t0 < 0 ? -t0 : 0;
            const int jhi = (g.T - t0) < g.k ? (g.T - t0) : g.k;
            lo = jlo * g.Cin - n0;
            hi = (rr < left) ? jhi * g.Cin - n0 : lo;
            if (hi > N - n0) hi = N - n0;
        };
    };
    Core<BM, BN, PA, PB> core;
    core.zero();
    pa.issue(arow(0));
    pb.issue(brow(0));
    pa.commit(lds);
    pb.commit(lds + PA::BYTES);
    __syncthreads();
    for (int st = 0; st < nsteps; ++st) {
        unsigned char* cur = lds + (st & 1) * STAGE;
        unsigned char* nxt = lds + ((st & 1) ^ 1) * STAGE;
        if (st + 1 < nsteps) { pa.issue(arow(st + 1)); pb.issue(brow(st + 1)); }
        core.step(cur, cur + PA::BYTES, wm, wn, lane);
        if (st + 1 < nsteps) { pa.commit(nxt); pb.commit(nxt + PA::BYTES); }
        __syncthreads();
    }
    core.for_each(wm, wn, lane, [&](int mm, int nn, float v) {
        const int m = m0 + mm, n = n0 + nn;
        if (m < M && n < N) {
            const size_t i = (size_t)m * N + n;
            dw[i] = accumulate ? dw[i] + v : v;
        }
    });
}

template <int BM, int BN, class PA, class PB>
constexpr int lds_bytes() { return 2 * (PA::BYTES + PB::BYTES); }

template <class K>
int set_lds(K kern, int bytes)
{
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    return W2L_OK;
}

// pick the tile whose grid wastes the fewest CU-rounds on a 256-CU part
struct TileChoice { int bm, bn; };
TileChoice choose_tile(long long M, long long N)
{
    const TileChoice cand[] = {{256, 256}, {192, 192}, {256, 128}, {128, 256}, {128, 128}};
    double best = -1;
    TileChoice pick = cand[0];
    for (const TileChoice& c : cand) {
        const long long tiles = ((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
        const long long rounds = (tiles + 255) / 256;
        // useful work / (rounds * 256 CUs * tile area), with a mild preference for big tiles
        double eff = (double)M * N / ((double)rounds * 256 * c.bm * c.bn);
        eff *= (c.bm * c.bn >= 192 * 192) ? 1.0 : (c.bm * c.bn >= 256 * 128 ? 0.95 : 0.85);
        if (eff > best) { best = eff; pick = c; }
    }
    return pick;
}

bool common_ok(int B, int T, int Cin, int Cout, int k, int s)
{
    if (Cin % 8 || Cout % 8) return false;
    if ((long long)k * Cin > 32767 * 8LL || (long long)k * Cout > 32767 * 8LL) return false;
    if ((long long)B * T * Cin >= (1LL << 31) || (long long)B * out_len(T, s) * Cout >= (1LL << 31)) return false;
    return true;
}

#define W2L_TILE_DISPATCH(CALL)                          \
    if (tc.bm == 256 && tc.bn == 256) { CALL(256, 256); } \
    else if (tc.bm == 192 && tc.bn == 192) { CALL(192, 192); } \
    else if (tc.bm == 256 && tc.bn == 128) { CALL(256, 128); } \
    else if (tc.bm == 128 && tc.bn == 256) { CALL(128, 256); } \
    else { CALL(128, 128); }

}  // namespace

bool conv_fwd_mfma_ok(int B, int T, int Cin, int Cout, int k, int s)
{
    return common_ok(B, T, Cin, Cout, k, s) && Cout >= 64 && (long long)B * out_len(T, s) >= 128;
}

int conv_fwd_mfma(const void* x, const void* w, const float* bias, void* y, int B, int T, int Cin, int Cout, int k,
                  int s, int ydt, hipStream_t st)
{
    ConvGeom g{B, T, out_len(T, s), Cin, Cout, k, s, (k - 1) / 2};
    const long long M = (long long)B * g.Tp, N = Cout;
    const TileChoice tc = choose_tile(M, N);
    int rc = W2L_OK;
#define CALL(BM_, BN_)                                                                                   \
    {                                                                                                    \
        constexpr int bytes = lds_bytes<BM_, BN_, PanelK<BM_>, PanelK<BN_>>();                           \
        const unsigned grid = (unsigned)(((M + BM_ - 1) / BM_) * ((N + BN_ - 1) / BN_));                 \
        if (ydt == W2L_BF16) {                                                                           \
            rc = set_lds(conv_fwd_k<BM_, BN_, bf16_t>, bytes);                                           \
            if (!rc) hipLaunchKernelGGL((conv_fwd_k<BM_, BN_, bf16_t>), dim3(grid), dim3(NT), bytes, st, \
                                        (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)y, g);        \
        } else {                                                                                         \
            rc = set_lds(conv_fwd_k<BM_, BN_, float>, bytes);                                            \
            if (!rc) hipLaunchKernelGGL((conv_fwd_k<BM_, BN_, float>), dim3(grid), dim3(NT), bytes, st,  \
                                        (const bf16_t*)x, (const bf16_t*)w, bias, (float*)y, g);         \
        }                                                                                                \
    }
    W2L_TILE_DISPATCH(CALL)
#undef CALL
    return rc ? rc : launch_status();
}

bool conv_dgrad_mfma_ok(int B, int T, int Cin, int Cout, int k, int s)
{
    return s == 1 && common_ok(B, T, Cin, Cout, k, s) && Cout % BK == 0 && Cin >= 64 && (long long)B * T >= 128;
}

int conv_dgrad_mfma(const void* dy, const void* w, void* dx, int B, int T, int Cin, int Cout, int k, int s,
                    hipStream_t st)
{
    ConvGeom g{B, T, out_len(T, s), Cin, Cout, k, s, (k - 1) / 2};
    const long long M = (long long)B * T, N = Cin;
    const TileChoice tc = choose_tile(M, N);
    int rc = W2L_OK;
#define CALL(BM_, BN_)                                                                               \
    {                                                                                                \
        constexpr int bytes = lds_bytes<BM_, BN_, PanelK<BM_>, PanelMN<BN_>>();                      \
        const unsigned grid = (unsigned)(((M + BM_ - 1) / BM_) * ((N + BN_ - 1) / BN_));             \
        rc = set_lds(conv_dgrad_k<BM_, BN_>, bytes);                                                 \
        if (!rc) hipLaunchKernelGGL((conv_dgrad_k<BM_, BN_>), dim3(grid), dim3(NT), bytes, st,       \
                                    (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, g);            \
    }
    W2L_TILE_DISPATCH(CALL)
#undef CALL
    return rc ? rc : launch_status();
}

bool conv_wgrad_mfma_ok(int B, int T, int Cin, int Cout, int k, int s)
{
    return common_ok(B, T, Cin, Cout, k, s) && Cout >= 64 && (long long)k * Cin >= 64;
}

size_t conv_wgrad_mfma_workspace(int, int, int, int, int, int) { return 0; }

int conv_wgrad_mfma(const void* x, const void* dy, float* dw, int B, int T, int Cin, int Cout, int k, int s,
                    int accumulate, void*, hipStream_t st)
{
    ConvGeom g{B, T, out_len(T, s), Cin, Cout, k, s, (k - 1) / 2};
    const long long M = Cout, N = (long long)k * Cin;
    const TileChoice tc = choose_tile(M, N);
    int rc = W2L_OK;
#define CALL(BM_, BN_)                                                                                \
    {                                                                                                 \
        constexpr int bytes = lds_bytes<BM_, BN_, PanelMN<BM_>, PanelMN<BN_>>();                      \
        const unsigned grid = (unsigned)(((M + BM_ - 1) / BM_) * ((N + BN_ - 1) / BN_));              \
        rc = set_lds(conv_wgrad_k<BM_, BN_>, bytes);                                                  \
        if (!rc) hipLaunchKernelGGL((conv_wgrad_k<BM_, BN_>), dim3(grid), dim3(NT), bytes, st,        \
                                    (const bf16_t*)x, (const bf16_t*)dy, dw, g, accumulate);          \
    }
    W2L_TILE_DISPATCH(CALL)
#undef CALL
    return rc ? rc : launch_status();
}

}  // namespace w2l
