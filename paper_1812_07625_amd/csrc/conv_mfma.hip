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
// One workgroup computes a BM x BN tile with one or two groups of 4 wavefronts (2x2).  Two
// groups put two wavefronts on every SIMD, which then work in opposite phases (one multiplies
// while the other moves data, see run_pingpong); each wavefront may then use 256 registers, i.e.
// hold a 96x96 or 128x64 block of accumulators.  The groups either split the reduction (KG = 2:
// alternate 16-element sub-steps of every panel, accumulators summed through LDS at the end;
// tiles up to 192x192 / 256x128) or the tile's columns (GN = 2: group g owns columns
// [g BN/2, (g+1) BN/2), tile 256x256).
//
// Data movement.  Operand panels of BKT reduction elements go global -> LDS directly
// (global_load_lds_dwordx4: no staging registers, no LDS store instructions) into a ring
// of STAGES panels, so the loads of panel st+STAGES-1 are in flight while panel st is
// multiplied; one barrier per panel.  Each load instruction fills 1 KB of LDS (lane i ->
// bytes 16i..16i+15), so the LDS image is dense; bank conflicts are avoided by an XOR
// swizzle of the 16-byte chunk index within each row, applied on the global-address
// side when loading and on the LDS-address side when reading.  r-contiguous panels are
// stored [row][BKT] and read with one 16-byte LDS read per MFMA operand; m/n-contiguous
// panels are stored [BKT][row] and read through the LDS transpose read
// (ds_read_b64_tr_b16), which hands each lane the 4 consecutive reduction elements of
// its row.  Zero padding at the utterance edges, ragged tiles and the reduction tail
// are handled by pointing the load of an out-of-range chunk at a 16-byte block of
// zeros (every lane always loads: the number of loads in flight is a constant, which
// the hand-placed s_waitcnt counts rely on); stores are predicated on the tile bounds.
//
// Two addressing modes.  CHECKED handles any caller tensor: per load, a range test picks the
// real address or the zero block.  FAST is for tensors laid out with a zero halo of at least
// (k-1)/2 frames around every utterance (the train step keeps its activations that way): every
// window is then plain in-bounds memory, the per-lane byte offsets are loop invariants, the
// panel advance is a scalar add on the base pointer, and a load costs three instructions.
#include <map>
#include <type_traits>
#include <mutex>
#include <utility>
#include "common.h"

namespace w2l {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) unsigned char lds_byte;


__device__ __align__(16) unsigned int g_zero16[4];  // source of every out-of-range chunk
// A row (1, 0, 0, ...) in bf16: the second operand of the weight gradient's extra column tile, whose first
// column is the bias gradient (sum of dy over the frames); every reduction row of that tile reads this row.
__device__ __align__(16) const unsigned short g_one_then_zeros[256] = {0x3F80};

typedef ConvDesc ConvGeom;

// 16 bytes per lane, global -> LDS at lds_addr + 16*lane (lds_addr wave-uniform).  Written
// as asm so that the compiler does not serialise later LDS reads behind it; completion is
// tracked by hand with wait_vmcnt<>.
__device__ __forceinline__ void dma16(const void* g, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr)
                 : "memory");
}
// same, address = uniform 64-bit base + per-lane 32-bit byte offset
__device__ __forceinline__ void dma16s(unsigned voff, const void* sbase, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// ---- r-contiguous panel: ROWS rows x BKT elements, dense [row][BKT] --------------------
// Row i of the tile is a run of memory starting at element offset off[i] (may point
// before the tensor for halo rows); reduction index r is valid in [lo, hi).
template <int ROWS, int BKT, int NW>
struct PanelK {
    static constexpr int ROWB = BKT * 2;               // bytes per LDS row
    static constexpr int BYTES = ROWS * ROWB;
    static constexpr int CPR = BKT / 8;                // 16-byte chunks per row
    static constexpr int RPB = 64 / CPR;               // rows filled by one load instruction
    static constexpr int NI = BYTES / 1024 / NW;       // load instructions per wavefront per panel
    static_assert(BYTES % (1024 * NW) == 0, "panel must split into 1 KB blocks over the wavefronts");
    static_assert(BKT == 64 || BKT == 32, "swizzles are written for 64- and 128-byte rows");
    int off[NI];                                       // element offsets (tensors hold < 2^31 elements)
    int lo[NI], hi[NI];                                // CHECKED mode only
    unsigned voff[NI];                                 // FAST mode only: byte offset of this lane's chunk at r0 = 0
    int c8;                                            // element offset inside a row of the chunk this lane loads
    const bf16_t* base;

    // chunk swizzle: rows that one LDS read instruction touches together land on distinct banks
    static __device__ __forceinline__ int swz(int row)
    {
        if (BKT == 64) return (row & 7) ^ ((row >> 3) & 1);
        return (((row >> 2) & 1) << 1) | (((row >> 1) ^ (row >> 3)) & 1);
    }
    static __device__ __forceinline__ int row_of(int i)
    {
        return ((threadIdx.x >> 6) + NW * i) * RPB + (threadIdx.x & 63) / CPR;
    }
    __device__ __forceinline__ void init(const bf16_t* b)
    {
        base = b;
        c8 = (((threadIdx.x & 63) % CPR) ^ swz(row_of(0))) * 8;  // swz(row_of(i)) is the same for every i
    }
    // load instruction i (of NI) of the panel whose first reduction index is r0, into the
    // stage at LDS address lds_stage
    __device__ __forceinline__ void issue(int i, int r0, unsigned lds_stage) const
    {
        const int r = r0 + c8;
        const unsigned wbase = __builtin_amdgcn_readfirstlane(lds_stage + (threadIdx.x >> 6) * 1024);
        const void* src = (r >= lo[i] && r < hi[i]) ? (const void*)(base + off[i] + r) : (const void*)g_zero16;
        dma16(src, wbase + i * (1024 * NW));
    }
    // FAST: row_off_elems = element offset of row i's reduction index 0 (always in bounds)
    __device__ __forceinline__ void set_fast(int i, long long row_off_elems) { voff[i] = (unsigned)((row_off_elems + c8) * 2); }
    __device__ __forceinline__ void issue_fast(int i, const bf16_t* sbase, unsigned lds_stage) const
    {
        const unsigned wbase = __builtin_amdgcn_readfirstlane(lds_stage + (threadIdx.x >> 6) * 1024);
        dma16s(voff[i], sbase, wbase + i * (1024 * NW));
    }
    // 32 rows starting at row0, sub-step ks (16 elements): lane holds row l%32, r = 8*(l/32)..+7
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int row0, int ks, int lane)
    {
        const int row = row0 + (lane & 31);
        const int slot = (2 * ks + (lane >> 5)) ^ swz(row);
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const s16x8*>(lds + row * ROWB + slot * 16));
    }
};

// ---- m/n-contiguous panel: BKT reduction rows x COLS elements, dense [BKT][COLS] --------
template <int COLS, int BKT, int NW>
struct PanelMN {
    static constexpr int RS = COLS * 2;
    static constexpr int BYTES = BKT * RS;
    static constexpr int CPR = COLS / 8;
    static constexpr int NI = BYTES / 1024 / NW;
    static_assert(BYTES % (1024 * NW) == 0, "panel must split into 1 KB blocks over the wavefronts");
    static_assert(CPR % 8 == 0, "the swizzle permutes chunks within aligned groups of 8 (or 16)");
    const bf16_t* base;
    // Chunk swizzle: the transpose read touches 4 consecutive reduction rows at once.  Rows that
    // are a multiple of 256 bytes apart start on the same bank, so all four need different chunk
    // groups (flip bits 2-3 with the row's low bits; needs CPR % 16 == 0); with 384-byte rows
    // (192 columns) only rows two apart collide, and flipping bit 2 with bit 1 of the row keeps
    // the permutation inside groups of 8 chunks.  swz(r + 4) == swz(r): the two reads of a
    // fragment share it.
    static __device__ __forceinline__ int swz(int row) { return CPR % 16 == 0 ? (row & 3) << 2 : ((row >> 1) & 1) << 2; }
    unsigned voff[NI];  // FAST mode only

    __device__ __forceinline__ void init(const bf16_t* b) { base = b; }
    // FAST: reduction row r of a panel starts row_pitch elements after row r-1; columns at or
    // beyond ncols are folded onto column 0 (their products land in outputs that are never stored)
    __device__ __forceinline__ void init_fast(const bf16_t* b, int row_pitch, int ncols)
    {
        base = b;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int q = chunk_of(i);
            const int row = q / CPR, slot = q - row * CPR;
            int c8 = (slot ^ swz(row)) * 8;
            if (c8 >= ncols) c8 = 0;
            voff[i] = (unsigned)(((long long)row * row_pitch + c8) * 2);
        }
    }
    __device__ __forceinline__ void issue_fast(int i, const bf16_t* sbase, unsigned lds_stage) const
    {
        const unsigned wbase = __builtin_amdgcn_readfirstlane(lds_stage + (threadIdx.x >> 6) * 1024);
        dma16s(voff[i], sbase, wbase + i * (1024 * NW));
    }
    static __device__ __forceinline__ int chunk_of(int i) { return ((threadIdx.x >> 6) + NW * i) * 64 + (threadIdx.x & 63); }
    // f(row, off, lo, hi): element offset of the row's column 0 of this tile and its valid
    // column range; the 16-byte chunk at column c is real data iff lo <= c < hi
    template <class F>
    __device__ __forceinline__ void issue(int i, F f, unsigned lds_stage) const
    {
        const unsigned wbase = __builtin_amdgcn_readfirstlane(lds_stage + (threadIdx.x >> 6) * 1024);
        const int q = chunk_of(i);
        const int row = q / CPR, slot = q - row * CPR;
        const int c8 = (slot ^ swz(row)) * 8;
        long long off;
        int lo, hi;
        f(row, off, lo, hi);
        const void* src = (c8 >= lo && c8 < hi) ? (const void*)(base + off + c8) : (const void*)g_zero16;
        dma16(src, wbase + i * (1024 * NW));
    }
    // Same fragment as PanelK::frag, gathered with two transpose reads: within each group of
    // 16 lanes, lane i supplies the address of row (i/4), columns 4*(i%4)..+3, and receives
    // column i of rows 0..3.
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int col0, int ks, int lane)
    {
        const int q = lane >> 4, i = lane & 15;
        const int col = col0 + 16 * (q & 1) + 4 * (i & 3);
        const int r = ks * 16 + 8 * (q >> 1) + (i >> 2);
        const int slot = (col >> 3) ^ swz(r);
        const unsigned char* p = lds + r * RS + slot * 16 + (col & 7) * 2;
        const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
        const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * RS));
        s16x8 v;
        v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
        v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
        return __builtin_bit_cast(bf16x8, v);
    }
};

// ---- the MFMA core: KG groups of 2x2 wavefronts ----------------------------------------
// Group kg multiplies the sub-steps ks = kg, kg + KG, ... of every panel.
template <int BM, int BN, int BKT, int KG, int GN, class PA, class PB>
struct Core {
    static_assert(KG * GN <= 2, "at most two groups of wavefronts");
    static constexpr int WTN = BN / (2 * GN);              // columns per wavefront (wn = 0 .. 2 GN - 1)
    static constexpr int TM = BM / 2 / 32, TN = WTN / 32;  // 32x32 blocks per wavefront
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
    // Operand fragments are double-buffered in registers: the LDS reads of this wavefront's next
    // sub-step are issued before the MFMAs of the current one, so their latency hides under
    // matrix work -- and this carries across panels: the first fragments of the next panel are
    // read before the last MFMAs of the current one.
    static constexpr int NS = BKT / 16 / KG;          // sub-steps per panel per wavefront
    static_assert(NS >= 2 && (BKT / 16) % KG == 0, "each group needs two sub-steps per panel to double-buffer");
    static constexpr int GROUPS = NS * TM * TN;      // MFMAs per panel per wavefront
    static constexpr int EARLY = (NS - 1) * TM * TN;  // MFMAs issued before the hand-over point
    bf16x8 fa[2][TM], fb[2][TN];
    // arow: row of the A panel that tile row 0 reads (non-zero when the panel is an activation slab)
    __device__ __forceinline__ void load_frags(int set, const unsigned char* la, const unsigned char* lb, int ks,
                                               int wm, int wn, int lane, int arow = 0)
    {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[set][i] = PA::frag(la, wm * (BM / 2) + i * 32 + arow, ks, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[set][j] = PB::frag(lb, wn * WTN + j * 32, ks, lane);
    }
    template <class Hook>
    __device__ __forceinline__ void mfmas(int u, Hook hook)
    {
        const int c = u & 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i], fb[c][j], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                hook((u * TM + i) * TN + j);
                __builtin_amdgcn_sched_barrier(0);
            }
    }
    // One panel whose first fragments (sub-step kg) are already in register set 0.  hook(g) runs
    // after this wavefront's g-th MFMA (the caller hangs the prefetch loads there, off the matrix
    // pipe's critical path); handover() runs before the last sub-step's MFMAs and must make the
    // next panel readable; the next panel's first fragments are then read from (na, nb) into set 0.
    template <class Hook, class Handover>
    __device__ __forceinline__ void step(const unsigned char* la, const unsigned char* lb, const unsigned char* na,
                                         const unsigned char* nb, int kg, int wm, int wn, int lane, Hook hook,
                                         Handover handover, int arow = 0, int narow = 0)
    {
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            if (u + 1 < NS) {
                load_frags((u + 1) & 1, la, lb, kg + KG * (u + 1), wm, wn, lane, arow);
            } else {
                handover();
                load_frags(0, na, nb, kg, wm, wn, lane, narow);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfmas(u, hook);
        }
    }
    // Ping-pong form (KG == 2): a wavefront first reads all its fragments of a panel, then
    // multiplies them; the two groups do this in opposite phases (see run_pingpong).
    __device__ __forceinline__ void read_panel(const unsigned char* la, const unsigned char* lb, int kg, int wm, int wn,
                                               int lane, int arow = 0)
    {
        static_assert(NS == 2, "one register set per sub-step");
#pragma unroll
        for (int u = 0; u < NS; ++u) load_frags(u, la, lb, kg + KG * u, wm, wn, lane, arow);
    }
    __device__ __forceinline__ void mfma_panel()
    {
#pragma unroll
        for (int u = 0; u < NS; ++u) mfmas(u, [](int) {});
    }
    // After reduce_groups() the finished sums of a tile are spread over both reduction groups: group 0 holds
    // the first OWN0 of a wavefront's TM x TN accumulator blocks, group 1 the rest -- so that the exchange
    // through LDS and all the epilogue work (rounding, staging, stores) run on all eight wavefronts.
    // Which blocks a group owns is a compile-time fact inside each of the two branches on the group (which is
    // uniform over a wavefront), so each branch is straight-line code over statically indexed registers.
    static constexpr int OWN0 = (TM * TN + 1) / 2;
    // group G owns blocks [LO<G>, HI<G>) of the wavefront's blocks in (i, j) row-major order
    template <int G> static constexpr int own_lo() { return (KG == 1 || G == 0) ? 0 : OWN0; }
    template <int G> static constexpr int own_hi() { return (KG == 1) ? TM * TN : (G == 0 ? OWN0 : TM * TN); }
    // The two branches on the group are the same code over different registers.  Left alone, the optimiser merges
    // them into one body that picks its registers by a run-time index -- which turns the accumulators into an
    // array in scratch memory.  A (comment-only) asm statement that differs between the branches, last in each,
    // keeps them apart.
    template <int G> static __device__ __forceinline__ void keep_apart()
    {
        if (G == 0) asm volatile("; reduction group 0" ::: "memory");
        else asm volatile("; reduction group 1" ::: "memory");
    }

    template <int G, class F>
    __device__ __forceinline__ void for_each_g(int wm, int wn, int lane, F f) const
    {
#pragma unroll
        for (int b = own_lo<G>(); b < own_hi<G>(); ++b) {
                const int i = b / TN, j = b % TN;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    f(m, wn * WTN + j * 32 + (lane & 31), acc[i][j][r], j);
                }
            }
        keep_apart<G>();
    }
    // f(m, n, value, j) for every element this lane holds and whose block its group owns; m,n relative to
    // the tile, j the element's column block within the wavefront
    template <class F>
    __device__ __forceinline__ void for_each(int kg, int wm, int wn, int lane, F f) const
    {
        if (KG == 1 || kg == 0) for_each_g<0>(wm, wn, lane, f);
        else for_each_g<1>(wm, wn, lane, f);
    }
    // bf16 output tile staged in LDS as [rows][BN] (rows padded by 16 bytes so that the two row
    // groups a wavefront writes at once fall on different banks): value + add[j], rounded.
    // Wavefront rows are taken relative to row_base.  Each group stages the blocks it owns.
    static constexpr int OPITCH = BN * 2 + 16;
    template <int G>
    __device__ __forceinline__ void stage_bf16_g(unsigned char* buf, const float (&add)[TN], int row_base, int wm, int wn,
                                                 int lane) const
    {
#pragma unroll
        for (int b = own_lo<G>(); b < own_hi<G>(); ++b) {
                const int i = b / TN, j = b % TN;
                const int n = wn * WTN + j * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3) - row_base;
                    *reinterpret_cast<bf16_t*>(buf + m * OPITCH + n * 2) = f32_to_bf16(acc[i][j][r] + add[j]);
                }
            }
        keep_apart<G>();
    }
    __device__ __forceinline__ void stage_bf16(unsigned char* buf, const float (&add)[TN], int row_base, int kg, int wm,
                                               int wn, int lane) const
    {
        if (KG == 1 || kg == 0) stage_bf16_g<0>(buf, add, row_base, wm, wn, lane);
        else stage_bf16_g<1>(buf, add, row_base, wm, wn, lane);
    }
    // KG == 2: each group hands the other, through LDS, its accumulators of the blocks the other owns and adds
    // what it receives to the blocks it owns (buf: 4 * TM * TN * 4 KB, free of panel traffic).  Lane-contiguous
    // 16-byte accesses; a sum has two terms, so its order is immaterial.
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    template <int G>
    __device__ __forceinline__ void hand_over(f32x4_t* q) const
    {
#pragma unroll
        for (int b = own_lo<1 - G>(); b < own_hi<1 - G>(); ++b) {
                const int i = b / TN, j = b % TN;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    f32x4_t v = {acc[i][j][4 * r4], acc[i][j][4 * r4 + 1], acc[i][j][4 * r4 + 2], acc[i][j][4 * r4 + 3]};
                    q[((i * TN + j) * 4 + r4) * 64] = v;
                }
            }
        keep_apart<G>();
    }
    template <int G>
    __device__ __forceinline__ void take_over(const f32x4_t* q)
    {
#pragma unroll
        for (int b = own_lo<G>(); b < own_hi<G>(); ++b) {
                const int i = b / TN, j = b % TN;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4_t v = q[((i * TN + j) * 4 + r4) * 64];
                    acc[i][j][4 * r4] += v[0];
                    acc[i][j][4 * r4 + 1] += v[1];
                    acc[i][j][4 * r4 + 2] += v[2];
                    acc[i][j][4 * r4 + 3] += v[3];
                }
            }
        keep_apart<G>();
    }
    __device__ __forceinline__ void reduce_groups(unsigned char* buf, int kg, int w4, int lane)
    {
        if (KG == 1) return;
        f32x4_t* q = reinterpret_cast<f32x4_t*>(buf) + (size_t)w4 * TM * TN * 4 * 64 + lane;
        __syncthreads();  // every wavefront has finished reading operand panels
        if (kg == 0) hand_over<0>(q);
        else hand_over<1>(q);
        __syncthreads();
        if (kg == 0) take_over<0>(q);
        else take_over<1>(q);
    }
    // The split data gradient's exchange between the two workgroups of a tile: the blocks this group owns go to
    // (come from) memory with device-scope cache policy (sc1: written through to, read from, memory).
    template <int G>
    __device__ __forceinline__ void store_owned_sc1(f32x4_t* mine) const
    {
#pragma unroll
        for (int b = own_lo<G>(); b < own_hi<G>(); ++b) {
                const int i = b / TN, j = b % TN;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4_t v = {acc[i][j][4 * r4], acc[i][j][4 * r4 + 1], acc[i][j][4 * r4 + 2], acc[i][j][4 * r4 + 3]};
                    f32x4_t* const dst = mine + (size_t)((i * TN + j) * 4 + r4) * 64;
                    // (the wait states: a store of more than 8 bytes reads its data registers a little after issue,
                    // and nothing tells the compiler's hazard check that this one does)
                    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(dst), "v"(v) : "memory");
                }
            }
        keep_apart<G>();
    }
    template <int G>
    __device__ __forceinline__ void add_owned_sc1(const f32x4_t* other)
    {
        // all of this group's blocks in flight together (at most OWN0 * 4 loads of 16 bytes per lane), one wait
        f32x4_t v[TM][TN][4];
#pragma unroll
        for (int b = own_lo<G>(); b < own_hi<G>(); ++b) {
                const int i = b / TN, j = b % TN;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4_t* const src = other + (size_t)((i * TN + j) * 4 + r4) * 64;
                    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v[i][j][r4]) : "v"(src) : "memory");
                }
            }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = own_lo<G>(); b < own_hi<G>(); ++b) {
                const int i = b / TN, j = b % TN;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    // tie each loaded register to the wait above: no use of it may be scheduled ahead of the wait
                    asm volatile("" : "+v"(v[i][j][r4])::"memory");
                    acc[i][j][4 * r4] += v[i][j][r4][0];
                    acc[i][j][4 * r4 + 1] += v[i][j][r4][1];
                    acc[i][j][4 * r4 + 2] += v[i][j][r4][2];
                    acc[i][j][4 * r4 + 3] += v[i][j][r4][3];
                }
            }
        keep_apart<G>();
    }
};

// The panel ring shared by the three kernels.  issue(i, p, lds_addr) starts load instruction
// i (of NL per wavefront) of panel p; for p >= nsteps it must load zeros or refetch valid data
// (the ring keeps prefetching past the end so that the number of loads in flight never changes).
//
// Per panel st, per wavefront, in program order:
//   MFMAs of all but the last sub-step, interleaved with the NL loads of panel st+STAGES-1 (they
//     go into the slot panel st-1 occupied; the barrier passed during panel st-1 freed it);
//   wait until this wavefront's loads of panel st+1 have landed, then barrier: now every
//     wavefront's share of panel st+1 is in LDS and nobody will read panel st again from
//     LDS (its last fragments are already in registers);
//   read the first fragments of panel st+1; MFMAs of the last sub-step of panel st.
template <int STAGES, int NL, int STAGE_BYTES, int A_BYTES, class CoreT, class Issue>
__device__ __forceinline__ void run_pipeline(CoreT& core, unsigned char* lds, int nsteps, Issue issue, int kg, int wm,
                                             int wn, int lane)
{
    static_assert(STAGES == 3 || STAGES == 4, "ring depth");
    static_assert((STAGES - 2) * NL < 64, "loads in flight must fit the vmcnt counter");
    // one load after every SPREAD-th MFMA: a burst of loads would fill the memory pipeline's
    // queue and stall the wavefront (and the MFMAs behind the load in program order) at issue
    constexpr int SPREAD = CoreT::GROUPS / NL;
    static_assert((NL - 1) * SPREAD < CoreT::GROUPS, "the prefetch loads must all be issued within the panel");
    // loads of the newest panel issued before the hand-over point
    constexpr int E = (CoreT::EARLY + SPREAD - 1) / SPREAD < NL ? (CoreT::EARLY + SPREAD - 1) / SPREAD : NL;
    const unsigned lds0 = (unsigned)(size_t)(lds_byte*)lds;
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) {
#pragma unroll
        for (int i = 0; i < NL; ++i) issue(i, s, lds0 + s * STAGE_BYTES);
    }
    wait_vmcnt<(STAGES - 2) * NL>();  // panel 0 has landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    core.load_frags(0, lds, lds + A_BYTES, kg, wm, wn, lane);
    int slot = 0;  // ring slot of panel st
    for (int st = 0; st < nsteps; ++st) {
        const int pre = st + STAGES - 1;
        int pslot = slot - 1;             // the slot panel st-1 occupied
        if (pslot < 0) pslot += STAGES;
        const int nslot = (slot + 1 == STAGES) ? 0 : slot + 1;
        const unsigned dst = lds0 + pslot * STAGE_BYTES;
        const unsigned char* cur = lds + slot * STAGE_BYTES;
        const unsigned char* nxt = lds + nslot * STAGE_BYTES;
        core.step(
            cur, cur + A_BYTES, nxt, nxt + A_BYTES, kg, wm, wn, lane,
            [&](int g) { if (g % SPREAD == 0 && g / SPREAD < NL) issue(g / SPREAD, pre, dst); },
            [&]() {
                // in flight, oldest first: panels st+1 .. st+STAGES-2 and the first E loads of
                // panel st+STAGES-1; panel st+1 must have landed
                wait_vmcnt<(STAGES - 3) * NL + E>();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wavefront's reads of panel st are done
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");  // no LDS read of panel st+1 may be hoisted above the barrier
            });
        slot = nslot;
    }
    wait_vmcnt<0>();  // the trailing panels must land before LDS is reused or released
}

// Ping-pong schedule for two groups of wavefronts (KG == 2).  Time is cut into phases with one
// workgroup barrier between consecutive phases.  In a "read" phase R(st) a wavefront starts its
// share of the loads of panel st+2, reads all its fragments of panel st from LDS and waits for
// its loads of panel st+1; in a "multiply" phase M(st) it only issues the MFMAs of panel st.
//     phase:    0      1      2      3      4    ...
//     group 0:  R(0)   M(0)   R(1)   M(1)   R(2) ...
//     group 1:  -      R(0)   M(0)   R(1)   M(1) ...
// so at any time one wavefront of every SIMD feeds the matrix pipe with nothing else in its
// instruction stream while the other does all the LDS and memory work -- LDS reads in the
// stream of a wavefront that is issuing MFMAs delay them, and two wavefronts that both
// multiply at once are served oldest-first, i.e. one after the other, with the pipe draining at
// every barrier.  Panel st is read in phases 2st and 2st+1; its ring slot is written again by
// loads issued in phase 2st+2 or later, and panel st+1 has landed (every wavefront waited for
// its own share at the end of a read phase no later than phase 2st+1) before phase 2st+2.
// grp = the group's phase offset (0 or 1); kg = which sub-steps of a panel the wavefront
// multiplies.  With a ring of STAGES slots the loads of panel st+STAGES-1 start in R(st).
template <int STAGES, int NL, int STAGE_BYTES, int A_BYTES, class CoreT, class Issue>
__device__ __forceinline__ void run_pingpong(CoreT& core, unsigned char* lds, int nsteps, Issue issue, int grp, int kg,
                                             int wm, int wn, int lane)
{
    static_assert(STAGES == 3 || STAGES == 4, "ring depth");
    static_assert((STAGES - 2) * NL < 64, "loads in flight must fit the vmcnt counter");
    const unsigned lds0 = (unsigned)(size_t)(lds_byte*)lds;
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) {
#pragma unroll
        for (int i = 0; i < NL; ++i) issue(i, s, lds0 + s * STAGE_BYTES);
    }
    wait_vmcnt<(STAGES - 2) * NL>();  // panel 0 has landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (grp == 1) {  // phase 0: nothing to do for group 1
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }
    int slot = 0;
    for (int st = 0; st < nsteps; ++st) {
        int pslot = slot - 1;  // the slot panel st-1 occupied = the slot of panel st+STAGES-1
        if (pslot < 0) pslot += STAGES;
        const unsigned dst = lds0 + pslot * STAGE_BYTES;
        const unsigned char* cur = lds + slot * STAGE_BYTES;
        // ---- R(st)
#pragma unroll
        for (int i = 0; i < NL; ++i) issue(i, st + STAGES - 1, dst);
        core.read_panel(cur, cur + A_BYTES, kg, wm, wn, lane);
        wait_vmcnt<(STAGES - 2) * NL>();                    // this wavefront's share of panel st+1 has landed
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // and its reads of panel st are done
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // ---- M(st)
        __builtin_amdgcn_sched_barrier(0);
        core.mfma_panel();
        __builtin_amdgcn_sched_barrier(0);
        if (grp == 0 || st + 1 < nsteps) {  // group 1's last multiply phase is the last phase
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        slot = (slot + 1 == STAGES) ? 0 : slot + 1;
    }
    wait_vmcnt<0>();  // the trailing panels must land before LDS is reused or released
}

template <int STAGES, int GROUPS, int NL, int STAGE_BYTES, int A_BYTES, class CoreT, class Issue>
__device__ __forceinline__ void run_ring(CoreT& core, unsigned char* lds, int nsteps, Issue issue, int grp, int kg, int wm,
                                         int wn, int lane)
{
    if constexpr (GROUPS == 2) {
        run_pingpong<STAGES, NL, STAGE_BYTES, A_BYTES>(core, lds, nsteps, issue, grp, kg, wm, wn, lane);
    } else {
        run_pipeline<STAGES, NL, STAGE_BYTES, A_BYTES>(core, lds, nsteps, issue, kg, wm, wn, lane);
    }
}

// The ring of the stride-1 forward / data-gradient passes when the A operand is kept as an
// activation slab: the reduction runs over channel blocks of 64 (outer) and taps (inner); the
// frames a tile needs from one channel block -- BM + k - 1 consecutive frames -- are loaded once
// into one of two slab buffers and serve all k taps (tap j reads the slab j rows further down),
// so only the weight panels stream through the three-slot ring, one per (channel block, tap).
// issue_slab(i, cb, lds_addr) starts load i (of NLS per wavefront) of channel block cb's slab;
// issue_b(i, cb, j, lds_addr) load i (of NLB) of the weight panel of (cb, j).  The slab of
// block cb+1 is requested in the read phase of the first panel of block cb, ahead of that
// phase's weight prefetch, so every wait that covers a weight panel also covers the older slab.
// Phases and barriers are those of run_pingpong.
template <int NLS, int NLB, int SLAB_BYTES, int STAGE_BYTES, class CoreT, class IssueSlab, class IssueB>
__device__ __forceinline__ void run_slab_pipeline(CoreT& core, unsigned char* lds, int ncb, int k, IssueSlab issue_slab,
                                                  IssueB issue_b, int kg, int wm, int wn, int lane)
{
    static_assert(NLS + NLB < 64, "loads in flight must fit the vmcnt counter");
    const unsigned lds0 = (unsigned)(size_t)(lds_byte*)lds;
    const unsigned ring0 = lds0 + 2 * SLAB_BYTES;
    unsigned char* ring = lds + 2 * SLAB_BYTES;
    const int nsteps = ncb * k;
    int pcb = 0, pj = 0;  // (channel block, tap) of the next weight panel to prefetch
    auto advance = [&]() {
        if (pj + 1 < k) ++pj;
        else if (pcb + 1 < ncb) { pj = 0; ++pcb; }  // past the end: keep refetching the last panel
    };
#pragma unroll
    for (int i = 0; i < NLS; ++i) issue_slab(i, 0, lds0);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < NLB; ++i) issue_b(i, pcb, pj, ring0 + s * STAGE_BYTES);
        advance();
    }
    wait_vmcnt<NLB>();  // slab 0 and weight panel 0 have landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kg == 1) {  // phase 0 of the ping-pong schedule: nothing to do for group 1
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }
    int cb = 0, j = 0, slot = 0;
    for (int st = 0; st < nsteps; ++st) {
        const bool has_slab = (j == 0) && (cb + 1 < ncb);
        int pslot = slot - 1;
        if (pslot < 0) pslot += 3;
        const unsigned dst = ring0 + pslot * STAGE_BYTES;
        const unsigned sdst = lds0 + ((cb + 1) & 1) * SLAB_BYTES;
        // ---- R(st): fragments first (the loads queue up behind each other in the memory pipeline
        // and would hold the reads back), then the slab of the next channel block (first tap only)
        // and weight panel st+2
        core.read_panel(lds + (cb & 1) * SLAB_BYTES, ring + slot * STAGE_BYTES, kg, wm, wn, lane, j);
        __builtin_amdgcn_sched_barrier(0);
        if (has_slab) {
#pragma unroll
            for (int i = 0; i < NLS; ++i) issue_slab(i, cb + 1, sdst);
        }
#pragma unroll
        for (int i = 0; i < NLB; ++i) issue_b(i, pcb, pj, dst);
        advance();
        // issued after weight panel st+1 (which must have landed): this phase's loads only
        if (has_slab) wait_vmcnt<NLS + NLB>();
        else wait_vmcnt<NLB>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // ---- M(st)
        __builtin_amdgcn_sched_barrier(0);
        core.mfma_panel();
        __builtin_amdgcn_sched_barrier(0);
        if (kg == 0 || st + 1 < nsteps) {
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        if (++j == k) { j = 0; ++cb; }
        slot = (slot + 1 == 3) ? 0 : slot + 1;
    }
    wait_vmcnt<0>();
}

// bf16 epilogue shared by the forward and data-gradient kernels: the accumulators (+ add[j] per
// column block) go to LDS as a row-major tile and leave as 16-byte row segments, every thread
// of the workgroup storing.  When the padded tile does not fit the panel ring (256x256) the
// two wavefront rows go one after the other.  rowoff(r) = output row (in units of N elements) of
// tile row r, negative for rows that must not be stored.
template <int BM, int BN, int NTHR, int LDS_BYTES, class CoreT, class RowOff>
__device__ __forceinline__ void store_tile_bf16(const CoreT& core, unsigned char* lds, const float (&add)[CoreT::TN],
                                                bf16_t* __restrict__ out, int n0, int N, int kg, int wm, int wn, int lane,
                                                RowOff rowoff)
{
    constexpr int PITCH = CoreT::OPITCH, CPRW = BN / 8;
    constexpr int PASSES = (BM * PITCH <= LDS_BYTES) ? 1 : 2;
    constexpr int ROWS = BM / PASSES;
    static_assert(ROWS * PITCH <= LDS_BYTES, "output tile staging must fit the panel ring");
    static_assert((ROWS * CPRW) % NTHR == 0, "row segments split evenly over the threads");
#pragma unroll
    for (int h = 0; h < PASSES; ++h) {
        __syncthreads();  // LDS is free: panels, group reduction or the previous pass are done with
        if (PASSES == 1 || wm == h) core.stage_bf16(lds, add, h * ROWS, kg, wm, wn, lane);
        __syncthreads();
#pragma unroll
        for (int c = threadIdx.x; c < ROWS * CPRW; c += NTHR) {
            const int row = c / CPRW, cc = c - row * CPRW;
            const int n = n0 + cc * 8;
            const long long ro = rowoff(h * ROWS + row);  // < 0: a row that is not stored
            if (ro >= 0 && n < N)
                *reinterpret_cast<uint4*>(out + (size_t)ro * N + n) =
                    *reinterpret_cast<const uint4*>(lds + row * PITCH + cc * 16);
        }
    }
}

// Workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its own
// L2); give each XCD a contiguous run of tiles, ordered with the shorter grid dimension
// fastest, so that the tiles sharing an L2 cover a compact block of operand panels -- or, with
// m_fastest, with the row tiles fastest, so that an XCD sees few column tiles and the weight
// slices it streams stay resident in its L2.
// xcd_m > 0 (chosen on the host, see xcd_split): the tile grid is cut into xcd_m x (8 / xcd_m)
// rectangular blocks, one per XCD, so that an L2 streams only its block's share of either operand;
// inside a block the column tiles run fastest.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn, bool m_fastest = false, int xcd_m = 0)
{
    if (xcd_m > 0) {
        const int xn = 8 / xcd_m, am = tiles_m / xcd_m, an = tiles_n / xn;
        const int x = blockIdx.x % 8, q = blockIdx.x / 8;
        tn = (x % xn) * an + q % an;
        tm = (x / xn) * am + q / an;
        return;
    }
    const int nb = tiles_m * tiles_n;
    const int per = (nb + 7) / 8;
    int id = (blockIdx.x % 8) * per + blockIdx.x / 8;
    if (nb % 8 != 0) id = blockIdx.x;  // keep it a bijection when the count does not split evenly
    if (tiles_n <= tiles_m && !m_fastest) { tm = id / tiles_n; tn = id % tiles_n; }
    else { tn = id / tiles_m; tm = id % tiles_m; }
}

// element offset of output row m = (b, t) in a tensor with `frames` frames per utterance
__device__ __forceinline__ long long out_row(int m, int frames, int pitch, int halo)
{
    if (pitch == frames && halo == 0) return m;
    const int b = m / frames;
    return (long long)b * pitch + halo + (m - b * frames);
}

// =============================== forward ================================================
template <int BM, int BN, int BKT, int STAGES, int KG, int GN, bool FAST, typename TO>
__global__ __launch_bounds__(256 * KG * GN) void conv_fwd_k(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                 const float* __restrict__ bias, TO* __restrict__ y, ConvGeom g)
{
    using PA = PanelK<BM, BKT, 4 * KG * GN>;
    using PB = PanelK<BN, BKT, 4 * KG * GN>;
    extern __shared__ __align__(1024) unsigned char lds[];
    constexpr int STAGE = PA::BYTES + PB::BYTES;
    static_assert(KG == 1 || BM * BN * 4 <= STAGES * STAGE, "the group reduction reuses the panel ring");
    const int M = g.B * g.Tp, N = g.Cout, K = g.k * g.Cin;
    int tm, tn;
    tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = wave >> 2, w4 = wave & 3, wm = w4 >> 1;
    const int kg = (KG == 2) ? grp : 0, wn = (GN == 2 ? 2 * grp : 0) + (w4 & 1);

    PA pa;
    PB pb;
    pa.init(x);
    pb.init(w);
#pragma unroll
    for (int i = 0; i < PA::NI; ++i) {
        int m = m0 + PA::row_of(i);
        if (FAST && m >= M) m = M - 1;                  // rows past the end recompute the last row; never stored
        const int b = m / g.Tp, tp = m - b * g.Tp;
        const int t0 = g.s * tp - g.p;                  // first frame of the window (may be < 0)
        const long long row = ((long long)b * g.x_pitch + g.x_halo + t0) * g.Cin;
        if (FAST) {
            pa.set_fast(i, row);
        } else {
            pa.off[i] = (int)row;
            pa.lo[i] = (t0 < 0 ? -t0 : 0) * g.Cin;
            const int last = g.T - t0;                  // taps j < last are inside the utterance
            pa.hi[i] = (m < M) ? (last < g.k ? last : g.k) * g.Cin : 0;
        }
    }
#pragma unroll
    for (int i = 0; i < PB::NI; ++i) {
        int n = n0 + PB::row_of(i);
        if (FAST) {
            if (n >= N) n = N - 1;
            pb.set_fast(i, (long long)n * K);
        } else {
            pb.off[i] = n * K;
            pb.lo[i] = 0;
            pb.hi[i] = (n < N) ? K : 0;
        }
    }
    Core<BM, BN, BKT, KG, GN, PA, PB> core;
    core.zero();
    const int nsteps = (K + BKT - 1) / BKT;  // FAST requires K % BKT == 0
    run_ring<STAGES, KG * GN, PA::NI + PB::NI, STAGE, PA::BYTES>(
        core, lds, nsteps,
        [&](int i, int st, unsigned dst) {
            if (FAST) {
                const int r0 = (st < nsteps ? st : nsteps - 1) * BKT;  // past the end: refetch the last panel
                if (i < PA::NI) pa.issue_fast(i, x + r0, dst);
                else pb.issue_fast(i - PA::NI, w + r0, dst + PA::BYTES);
            } else {
                if (i < PA::NI) pa.issue(i, st * BKT, dst);
                else pb.issue(i - PA::NI, st * BKT, dst + PA::BYTES);
            }
        },
        grp, kg, wm, wn, lane);
    core.reduce_groups(lds, kg, w4, lane);
    float bv[core.TN];
#pragma unroll
    for (int j = 0; j < core.TN; ++j) {
        const int n = n0 + wn * core.WTN + j * 32 + (lane & 31);
        bv[j] = (bias && n < N) ? bias[n] : 0.f;
    }
    if (sizeof(TO) == 2 && N % 8 == 0) {
        store_tile_bf16<BM, BN, 256 * KG * GN, STAGES * STAGE>(
            core, lds, bv, reinterpret_cast<bf16_t*>(y), n0, N, kg, wm, wn, lane,
            [&](int r) { return m0 + r < M ? out_row(m0 + r, g.Tp, g.y_pitch, g.y_halo) : -1LL; });
        return;
    }
    core.for_each(kg, wm, wn, lane, [&](int mm, int nn, float v, int j) {
        const int m = m0 + mm, n = n0 + nn;
        if (m < M && n < N) Elem<TO>::store(y, (size_t)out_row(m, g.Tp, g.y_pitch, g.y_halo) * N + n, v + bv[j]);
    });
}

// dynamic LDS of a slab kernel: two slabs + three weight panels, or the fp32 tile of the group reduction
constexpr int slab_lds_bytes(int bm, int bn, int srows, int kg)
{
    const int ring = 2 * srows * 128 + 3 * bn * 128;
    return (kg == 2 && bm * bn * 4 > ring) ? bm * bn * 4 : ring;
}

// Forward pass, stride 1, input kept with a zero halo (see FAST above), Cin % 64 == 0: tiles
// run over the frames of the input *layout* (halo frames included; their outputs are dropped),
// so that the frames a tile reads are one contiguous block -- the activation slab.
// GLUF: the layer's GLU is applied in the epilogue.  The tile then takes its first BN/2 columns
// from the value half of the output channels and the other BN/2 from the matching gate channels
// (column c of the tile <-> channel chan(c)), so that both operands of every GLU output sit in
// the same staged tile; besides y it writes h = a * sigmoid(g) ([frames][Cout/2], the time layout
// of x, zeros in halo frames and in the zeroed part of the slack).
template <int BM, int BN, int SROWS, int KG, typename TO, bool GLUF>
__global__ __launch_bounds__(256 * KG) void conv_fwd_slab_k(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                            const float* __restrict__ bias, TO* __restrict__ y,
                                                            bf16_t* __restrict__ h, ConvGeom g)
{
    using PS = PanelK<SROWS, 64, 4 * KG>;
    using PB = PanelK<BN, 64, 4 * KG>;
    extern __shared__ __align__(1024) unsigned char lds[];
    constexpr int LDS_BYTES = slab_lds_bytes(BM, BN, SROWS, KG);
    const int F = (g.B - 1) * g.x_pitch + g.T;  // frames from the first real one to the last real one
    const int N = g.Cout, K = g.k * g.Cin, H = g.Cout / 2;
    const int tiles_m = (F + BM - 1) / BM;
    int tm, tn;
    tile_of_block(tiles_m, (N + BN - 1) / BN, tm, tn, false, g.xcd_m);
    const int f0 = g.x_halo + tm * BM, n0 = tn * BN;  // layout frame of tile row 0
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kg = wave >> 2, w4 = wave & 3, wm = w4 >> 1, wn = w4 & 1;
    // output channel of tile column c (GLUF requires H % (BN/2) == 0, so no tile is ragged)
    auto chan = [&](int c) { return GLUF ? (c < BN / 2 ? tn * (BN / 2) + c : H + tn * (BN / 2) + c - BN / 2) : n0 + c; };

    PS ps;
    PB pb;
    ps.init(x);
    pb.init(w);
#pragma unroll
    for (int i = 0; i < PS::NI; ++i) ps.set_fast(i, (long long)(f0 - g.p + PS::row_of(i)) * g.Cin);
#pragma unroll
    for (int i = 0; i < PB::NI; ++i) {
        int n = chan(PB::row_of(i));
        if (n >= N) n = N - 1;
        pb.set_fast(i, (long long)n * K);
    }
    Core<BM, BN, 64, KG, 1, PS, PB> core;
    core.zero();
    run_slab_pipeline<PS::NI, PB::NI, PS::BYTES, PB::BYTES>(
        core, lds, g.Cin / 64, g.k,
        [&](int i, int cb, unsigned dst) { ps.issue_fast(i, x + cb * 64, dst); },
        [&](int i, int cb, int j, unsigned dst) { pb.issue_fast(i, w + (j * g.Cin + cb * 64), dst); }, kg, wm, wn, lane);
    core.reduce_groups(lds, kg, w4, lane);
    float bv[core.TN];
#pragma unroll
    for (int j = 0; j < core.TN; ++j) {
        const int n = chan(wn * core.WTN + j * 32 + (lane & 31));
        bv[j] = (bias && n < N) ? bias[n] : 0.f;
    }
    // tile row r is layout frame f0 + r: utterance b, frame t; stored only if it is a real frame
    auto rowoff = [&](int r) {
        const int f = f0 + r, b = f / g.x_pitch, t = f - b * g.x_pitch - g.x_halo;
        return (b < g.B && t >= 0 && t < g.T) ? (long long)b * g.y_pitch + g.y_halo + t : -1LL;
    };
    if constexpr (GLUF) {
        static_assert(sizeof(TO) == 2, "the fused GLU writes bf16");
        constexpr int PITCH = core.OPITCH, CPH = BN / 16, NTHR = 256 * KG;  // CPH: 16-byte chunks per half row
        static_assert(BM * PITCH <= LDS_BYTES, "output tile staging");
        bf16_t* yo = reinterpret_cast<bf16_t*>(y);
        __syncthreads();
        core.stage_bf16(lds, bv, 0, kg, wm, wn, lane);
        __syncthreads();
        const long long zero_end = (long long)g.B * g.x_pitch + LAYOUT_SLACK_ZERO;  // h is zero up to here outside real frames
        const int ch0 = tn * (BN / 2);
#pragma unroll 2
        for (int c = threadIdx.x; c < BM * CPH; c += NTHR) {
            const int row = c / CPH, cc = c - row * CPH;
            const int f = f0 + row;
            const long long ro = rowoff(row);
            uint4 oh = make_uint4(0, 0, 0, 0);
            if (ro >= 0) {
                const uint4 ua = *reinterpret_cast<const uint4*>(lds + row * PITCH + cc * 16);
                const uint4 ug = *reinterpret_cast<const uint4*>(lds + row * PITCH + (BN / 2) * 2 + cc * 16);
                *reinterpret_cast<uint4*>(yo + (size_t)ro * N + ch0 + cc * 8) = ua;
                *reinterpret_cast<uint4*>(yo + (size_t)ro * N + H + ch0 + cc * 8) = ug;
                const unsigned* pa = &ua.x; const unsigned* pg = &ug.x;
                unsigned* qh = &oh.x;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    unsigned r2 = 0;
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const float a = bf16_to_f32((bf16_t)(pa[q] >> (16 * hh)));
                        const float gg = bf16_to_f32((bf16_t)(pg[q] >> (16 * hh)));
                        r2 |= (unsigned)f32_to_bf16(a * sigmoidf_(gg)) << (16 * hh);
                    }
                    qh[q] = r2;
                }
            }
            if (f < zero_end || ro >= 0) *reinterpret_cast<uint4*>(h + (size_t)f * H + ch0 + cc * 8) = oh;
        }
        // frames no tile covers: the leading halo (first row of tiles) and from the end of the last
        // tile to the end of the zeroed slack (last row of tiles)
        const long long t_end = (long long)g.x_halo + (long long)tiles_m * BM;
        const long long lead = (tm == 0) ? g.x_halo : 0, trail = (tm == tiles_m - 1 && t_end < zero_end) ? zero_end - t_end : 0;
        for (long long c = threadIdx.x; c < (lead + trail) * CPH; c += NTHR) {
            const long long r = c / CPH;
            const int cc = (int)(c - r * CPH);
            const long long f = r < lead ? r : t_end + (r - lead);
            *reinterpret_cast<uint4*>(h + (size_t)f * H + ch0 + cc * 8) = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    if (sizeof(TO) == 2 && N % 8 == 0) {
        store_tile_bf16<BM, BN, 256 * KG, LDS_BYTES>(core, lds, bv, reinterpret_cast<bf16_t*>(y), n0, N, kg, wm, wn, lane, rowoff);
        return;
    }
    core.for_each(kg, wm, wn, lane, [&](int mm, int nn, float v, int j) {
        const long long ro = rowoff(mm);
        const int n = n0 + nn;
        if (ro >= 0 && n < N) Elem<TO>::store(y, (size_t)ro * N + n, v + bv[j]);
    });
}

// =============================== data gradient (stride 1) =============================
// dx[b,t,ci] = sum_{j',co} dy[b, t-p+j', co] * w[co, k-1-j', ci]
template <int BM, int BN, int BKT, int STAGES, int KG, int GN, bool FAST>
__global__ __launch_bounds__(256 * KG * GN) void conv_dgrad_k(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ w,
                                                   bf16_t* __restrict__ dx, ConvGeom g)
{
    using PA = PanelK<BM, BKT, 4 * KG * GN>;
    using PB = PanelMN<BN, BKT, 4 * KG * GN>;
    extern __shared__ __align__(1024) unsigned char lds[];
    constexpr int STAGE = PA::BYTES + PB::BYTES;
    static_assert(KG == 1 || BM * BN * 4 <= STAGES * STAGE, "the group reduction reuses the panel ring");
    const int M = g.B * g.T, N = g.Cin, K = g.k * g.Cout;
    int tm, tn;
    tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = wave >> 2, w4 = wave & 3, wm = w4 >> 1;
    const int kg = (KG == 2) ? grp : 0, wn = (GN == 2 ? 2 * grp : 0) + (w4 & 1);

    PA pa;
    PB pb;
    pa.init(dy);
    if (FAST) pb.init_fast(w, g.k * g.Cin, N - n0);
    else pb.init(w);
#pragma unroll
    for (int i = 0; i < PA::NI; ++i) {
        int m = m0 + PA::row_of(i);
        if (FAST && m >= M) m = M - 1;
        const int b = m / g.T, t = m - b * g.T;
        const int t0 = t - g.p;
        const long long row = ((long long)b * g.y_pitch + g.y_halo + t0) * g.Cout;
        if (FAST) {
            pa.set_fast(i, row);
        } else {
            pa.off[i] = (int)row;
            pa.lo[i] = (t0 < 0 ? -t0 : 0) * g.Cout;
            const int last = g.Tp - t0;
            pa.hi[i] = (m < M) ? (last < g.k ? last : g.k) * g.Cout : 0;
        }
    }
    Core<BM, BN, BKT, KG, GN, PA, PB> core;
    core.zero();
    const int nsteps = K / BKT;  // Cout is a multiple of BKT: a panel stays inside one tap
    run_ring<STAGES, KG * GN, PA::NI + PB::NI, STAGE, PA::BYTES>(
        core, lds, nsteps,
        [&](int i, int st, unsigned dst) {
            const int stc = (FAST && st >= nsteps) ? nsteps - 1 : st;
            const int r0 = stc * BKT;
            if (i < PA::NI) {
                if (FAST) pa.issue_fast(i, dy + r0, dst);
                else pa.issue(i, r0, dst);
                return;
            }
            const int jp = r0 / g.Cout, co0 = r0 - jp * g.Cout;
            const long long tapoff = (long long)(g.k - 1 - jp) * g.Cin + n0;
            if (FAST) {
                pb.issue_fast(i - PA::NI, w + (long long)co0 * g.k * g.Cin + tapoff, dst + PA::BYTES);
                return;
            }
            const int ncols = N - n0;
            pb.issue(i - PA::NI,
                [=](int rr, long long& off, int& lo, int& hi) {
                    off = (long long)(co0 + rr) * g.k * g.Cin + tapoff;
                    lo = 0;
                    hi = (st < nsteps) ? ncols : 0;  // chunk columns are multiples of 8 and N % 8 == 0
                },
                dst + PA::BYTES);
        },
        grp, kg, wm, wn, lane);
    core.reduce_groups(lds, kg, w4, lane);
    float zero[core.TN];
#pragma unroll
    for (int j = 0; j < core.TN; ++j) zero[j] = 0.f;
    store_tile_bf16<BM, BN, 256 * KG * GN, STAGES * STAGE>(
        core, lds, zero, dx, n0, N, kg, wm, wn, lane,
        [&](int r) { return m0 + r < M ? out_row(m0 + r, g.T, g.x_pitch, g.x_halo) : -1LL; });
}

// Data gradient with the dy window kept as an activation slab (dy has a zero halo, Cout % 64
// == 0): same schedule as conv_fwd_slab_k; the weight panel of (channel block, tap j') is the
// 64 x BN block w[co0 .. co0+63][k-1-j'][n0 .. n0+BN-1], read through the LDS transpose read.
// GLUB: the tile is not stored as dx but pushed through the GLU backward of the layer below
// (whose pre-GLU activations yprev are dense [B*T, 2N]): dx_out then has 2N channels and the
// time layout of dy (tile row r -> its frame f0 + r); frames that are not real get zeros.
// part != nullptr (grid.y = 2): the reduction over channel blocks is split in two between the two
// workgroups (blockIdx.y) of a tile -- twice the workgroups when one per tile leaves CUs idle.  Each
// stores its fp32 sums to its own slot of `part` and then takes a ticket from the tile's counter
// (zeroed before the launch); the one that draws the second ticket adds the other's sums to its own
// and finishes the tile.  Nobody waits for anybody, and since a + b == b + a the result does not
// depend on which of the two comes second.  The slots hold the accumulators in register order
// ([wavefront][accumulator quad][lane], 16 bytes per lane: both workgroups map threads to elements
// alike), so every store and load instruction moves 1 KB of consecutive memory.
template <int BM, int BN, int SROWS, int KG, bool GLUB>
__global__ __launch_bounds__(256 * KG) void conv_dgrad_slab_k(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ w,
                                                              bf16_t* __restrict__ dx, const bf16_t* __restrict__ yprev,
                                                              float* __restrict__ part, int* __restrict__ tickets, ConvGeom g)
{
    using PS = PanelK<SROWS, 64, 4 * KG>;
    using PB = PanelMN<BN, 64, 4 * KG>;
    extern __shared__ __align__(1024) unsigned char lds[];
    constexpr int LDS_BYTES = slab_lds_bytes(BM, BN, SROWS, KG);
    const int F = (g.B - 1) * g.y_pitch + g.Tp;
    const int N = g.Cin;
    int tm, tn, half = 0;
    const int tiles_m = (F + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    if (part && g.xcd_m > 0) {
        // split reduction, 1-D grid of 2 * tiles workgroups: an XCD takes one half of the reduction (its parity)
        // of one of xcd_m x (4 / xcd_m) rectangular blocks of tiles, so its L2 streams only that block's rows of
        // dy and columns of w, and of those only its half of the channel blocks
        const int x = blockIdx.x % 8, q = blockIdx.x / 8, blk = x >> 1;
        const int xn = 4 / g.xcd_m, am = tiles_m / g.xcd_m, an = tiles_n / xn;
        half = x & 1;
        tn = (blk % xn) * an + q % an;
        tm = (blk / xn) * am + q / an;
    } else {
        tile_of_block(tiles_m, tiles_n, tm, tn, true);
        half = blockIdx.y;
    }
    const int f0 = g.y_halo + tm * BM, n0 = tn * BN;  // dy layout frame of tile row 0
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kg = wave >> 2, w4 = wave & 3, wm = w4 >> 1, wn = w4 & 1;

    PS ps;
    PB pb;
    ps.init(dy);
    pb.init_fast(w, g.k * g.Cin, N - n0);
#pragma unroll
    for (int i = 0; i < PS::NI; ++i) ps.set_fast(i, (long long)(f0 - g.p + PS::row_of(i)) * g.Cout);
    Core<BM, BN, 64, KG, 1, PS, PB> core;
    core.zero();
    const int nparts = part ? 2 : 1, ncb = g.Cout / 64 / nparts, cb0 = half * ncb;  // this workgroup's channel blocks
    run_slab_pipeline<PS::NI, PB::NI, PS::BYTES, PB::BYTES>(
        core, lds, ncb, g.k,
        [&](int i, int cb, unsigned dst) { ps.issue_fast(i, dy + (cb0 + cb) * 64, dst); },
        [&](int i, int cb, int j, unsigned dst) {
            pb.issue_fast(i, w + ((long long)(cb0 + cb) * 64 * g.k + (g.k - 1 - j)) * g.Cin + n0, dst);
        },
        kg, wm, wn, lane);
    core.reduce_groups(lds, kg, w4, lane);
    if (part) {
        typedef __attribute__((ext_vector_type(4))) float f32x4;
        constexpr int QUADS = core.TM * core.TN * 4;                       // 16-byte pieces per lane
        constexpr size_t SLOT = (size_t)4 * QUADS * 64;                    // f32x4 per workgroup slot
        const int tile = tm * tiles_n + tn;
        f32x4* mine = reinterpret_cast<f32x4*>(part) + ((size_t)tile * 2 + half) * SLOT + ((size_t)w4 * QUADS) * 64 + lane;
        const f32x4* other = reinterpret_cast<const f32x4*>(part) + ((size_t)tile * 2 + (1 - half)) * SLOT + ((size_t)w4 * QUADS) * 64 + lane;
        // The sums cross from one XCD's L2 to another's: they are stored and loaded with device-scope
        // cache policy (sc1: written through to, and read from, memory), and each side waits for its
        // own accesses to complete around the ticket -- no cache-wide write-back or invalidate, which
        // would throw out the operand panels the other workgroups of this L2 are streaming.
        // (each reduction group stores, and later loads, the accumulator blocks it owns)
        if (kg == 0) core.template store_owned_sc1<0>(mine);
        else core.template store_owned_sc1<1>(mine);
        wait_vmcnt<0>();   // this thread's sums have reached memory
        __syncthreads();   // ... and every thread's
        int* ticket_lds = reinterpret_cast<int*>(lds);  // the panel ring is free by now
        if (threadIdx.x == 0) *ticket_lds = __hip_atomic_fetch_add(tickets + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int ticket = *ticket_lds;
        if (ticket == 0) return;  // first of the pair: the other workgroup finishes the tile
        if (kg == 0) core.template add_owned_sc1<0>(other);
        else core.template add_owned_sc1<1>(other);
    }
    float zero[core.TN];
#pragma unroll
    for (int j = 0; j < core.TN; ++j) zero[j] = 0.f;
    if (!GLUB) {
        store_tile_bf16<BM, BN, 256 * KG, LDS_BYTES>(core, lds, zero, dx, n0, N, kg, wm, wn, lane, [&](int r) {
            const int f = f0 + r, b = f / g.y_pitch, t = f - b * g.y_pitch - g.y_halo;
            return (b < g.B && t >= 0 && t < g.T) ? (long long)b * g.x_pitch + g.x_halo + t : -1LL;
        });
        return;
    }
    // dh tile (rounded to bf16, as the unfused path stores it) -> LDS -> GLU backward, 8 channels per thread
    constexpr int PITCH = core.OPITCH, CPRW = BN / 8, NTHR = 256 * KG;
    static_assert(BM * PITCH <= LDS_BYTES && (BM * CPRW) % NTHR == 0, "dh tile staging");
    __syncthreads();
    core.stage_bf16(lds, zero, 0, kg, wm, wn, lane);
    __syncthreads();
    const long long alloc_frames = (long long)g.B * g.y_pitch + g.slack;
#pragma unroll 2
    for (int c = threadIdx.x; c < BM * CPRW; c += NTHR) {
        const int row = c / CPRW, cc = c - row * CPRW;
        const int n = n0 + cc * 8;
        const int f = f0 + row, b = f / g.y_pitch, t = f - b * g.y_pitch - g.y_halo;
        if (n >= N || f >= alloc_frames) continue;
        uint4 oa = make_uint4(0, 0, 0, 0), og = oa;
        if (b < g.B && t >= 0 && t < g.T) {
            const bf16_t* yr = yprev + ((size_t)b * g.T + t) * 2 * N + n;
            const uint4 ua = *reinterpret_cast<const uint4*>(yr), ug = *reinterpret_cast<const uint4*>(yr + N);
            const uint4 ud = *reinterpret_cast<const uint4*>(lds + row * PITCH + cc * 16);
            const unsigned* pa = &ua.x; const unsigned* pg = &ug.x; const unsigned* pd = &ud.x;
            unsigned* qa = &oa.x; unsigned* qg = &og.x;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned ra = 0, rg = 0;
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const float a = bf16_to_f32((bf16_t)(pa[q] >> (16 * hh)));
                    const float gg = bf16_to_f32((bf16_t)(pg[q] >> (16 * hh)));
                    const float d = bf16_to_f32((bf16_t)(pd[q] >> (16 * hh)));
                    const float sg = sigmoidf_(gg);
                    ra |= (unsigned)f32_to_bf16(d * sg) << (16 * hh);
                    rg |= (unsigned)f32_to_bf16(d * a * sg * (1.f - sg)) << (16 * hh);
                }
                qa[q] = ra;
                qg[q] = rg;
            }
        }
        bf16_t* o = dx + (size_t)f * 2 * N + n;
        *reinterpret_cast<uint4*>(o) = oa;
        *reinterpret_cast<uint4*>(o + N) = og;
    }
}

// zero rows [r0, r1) and [r2, r3) of a [rows, C] bf16 tensor (C % 8 == 0), and n_tickets ints
__global__ __launch_bounds__(256) void zero_rows_k(bf16_t* __restrict__ p, long long r0, long long r1, long long r2,
                                                   long long r3, int C, int* __restrict__ tickets, int n_tickets)
{
    const int cv = C / 8;
    const long long na = (r1 - r0) * cv, nb = (r3 - r2) * cv;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < na + nb; i += (long long)gridDim.x * blockDim.x) {
        const long long e = i < na ? r0 * cv + i : r2 * cv + (i - na);
        reinterpret_cast<uint4*>(p)[e] = make_uint4(0, 0, 0, 0);
    }
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_tickets; i += gridDim.x * blockDim.x) tickets[i] = 0;
}

// =============================== weight gradient ========================================
// dw[co, (j,ci)] = sum_{b,t'} dy[b,t',co] * x[b, s t' - p + j, ci].
// CHECKED: the reduction walks utterance by utterance in BKT-frame panels (the last panel of
// an utterance is masked).  FAST (stride 1, x and dy share one haloed time layout): the
// reduction runs straight through the frames of all utterances including the halo frames
// between them -- dy is zero there, so they add nothing -- which makes every panel a dense
// block of BKT consecutive frames of both tensors.
// FAST with dbias != nullptr: the grid has one more column of tiles.  Its second operand is the constant
// row (1, 0, 0, ...) for every frame, so its first output column is sum_t dy[t, co] -- the bias
// gradient -- computed by the same pipeline with the same loads per phase, in a fixed order.
template <int BM, int BN, int BKT, int STAGES, int KG, int GN, bool FAST, bool BIAS>
__global__ __launch_bounds__(256 * KG * GN) void conv_wgrad_k(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                   float* __restrict__ dw, float* __restrict__ dbias, ConvGeom g, int accumulate)
{
    static_assert(FAST || !BIAS, "the bias column rides on the dense walk through the frames");
    using PA = PanelMN<BM, BKT, 4 * KG * GN>;
    using PB = PanelMN<BN, BKT, 4 * KG * GN>;
    extern __shared__ __align__(1024) unsigned char lds[];
    constexpr int STAGE = PA::BYTES + PB::BYTES;
    static_assert(KG == 1 || BM * BN * 4 <= STAGES * STAGE, "the group reduction reuses the panel ring");
    const int M = g.Cout, N = g.w_cols ? g.w_cols : g.k * g.Cin;
    const int tiles_n = (N + BN - 1) / BN;
    int tm, tn;
    tile_of_block((M + BM - 1) / BM, tiles_n + (BIAS ? 1 : 0), tm, tn);
    const bool bias_tile = BIAS && tn == tiles_n;  // uniform over the workgroup
    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = wave >> 2, w4 = wave & 3, wm = w4 >> 1;
    const int kg = (KG == 2) ? grp : 0, wn = (GN == 2 ? 2 * grp : 0) + (w4 & 1);
    const bf16_t* const ones = reinterpret_cast<const bf16_t*>(g_one_then_zeros);
    static_assert(BN <= 256, "the constant row covers one tile width");

    PA pa;
    PB pb;
    if (FAST) {
        pa.init_fast(dy, g.Cout, M - m0);
        if (bias_tile) pb.init_fast(ones, 0, BN);  // row pitch 0: every reduction row is the same row
        else pb.init_fast(x, g.Cin, N - n0);
    } else {
        pa.init(dy);
        pb.init(x);
    }
    const int spb = (g.Tp + BKT - 1) / BKT;  // CHECKED: panels per utterance
    const int frames = (g.B - 1) * g.y_pitch + g.Tp;  // FAST: first real frame of utterance 0 .. last real frame
    const int nsteps = FAST ? (frames + BKT - 1) / BKT : g.B * spb;
    Core<BM, BN, BKT, KG, GN, PA, PB> core;
    core.zero();
    run_ring<STAGES, KG * GN, PA::NI + PB::NI, STAGE, PA::BYTES>(
        core, lds, nsteps,
        [&](int i, int st, unsigned dst) {
            if (FAST) {
                const long long f0 = (long long)(st < nsteps ? st : nsteps - 1) * BKT;
                if (i < PA::NI) pa.issue_fast(i, dy + (g.y_halo + f0) * g.Cout + m0, dst);
                else pb.issue_fast(i - PA::NI, bias_tile ? ones : x + (g.x_halo - g.p + f0) * g.Cin + n0, dst + PA::BYTES);
                return;
            }
            const int b = st / spb, tp0 = (st - b * spb) * BKT;
            const int left = (st < nsteps) ? g.Tp - tp0 : 0;  // past the end: every row masked
            if (i < PA::NI) {
                const long long boff = ((long long)b * g.y_pitch + g.y_halo + tp0) * g.Cout + m0;
                const int mcols = M - m0;
                pa.issue(i,
                    [=](int rr, long long& off, int& lo, int& hi) {
                        off = boff + (long long)rr * g.Cout;
                        lo = 0;
                        hi = (rr < left) ? mcols : 0;
                    },
                    dst);
                return;
            }
            pb.issue(i - PA::NI,
                [=](int rr, long long& off, int& lo, int& hi) {
                    const int t0 = g.s * (tp0 + rr) - g.p;          // frame under tap 0
                    off = ((long long)b * g.x_pitch + g.x_halo + t0) * g.Cin + n0;
                    // tile column c <-> tap-major index n0 + c ; valid taps: 0 <= t0 + j < T
                    const int jlo = t0 < 0 ? -t0 : 0;
                    const int jhi = (g.T - t0) < g.k ? (g.T - t0) : g.k;
                    lo = jlo * g.Cin - n0;
                    hi = (rr < left) ? jhi * g.Cin - n0 : lo;
                    if (hi > N - n0) hi = N - n0;
                },
                dst + PA::BYTES);
        },
        grp, kg, wm, wn, lane);
    core.reduce_groups(lds, kg, w4, lane);
    if (bias_tile) {
        core.for_each(kg, wm, wn, lane, [&](int mm, int nn, float v, int) {
            const int m = m0 + mm;
            if (nn == 0 && m < M) dbias[m] = accumulate ? dbias[m] + v : v;
        });
        return;
    }
    core.for_each(kg, wm, wn, lane, [&](int mm, int nn, float v, int) {
        const int m = m0 + mm, n = n0 + nn;
        if (m < M && n < N) {
            const size_t i = (size_t)m * N + n;
            __builtin_nontemporal_store(accumulate ? dw[i] + v : v, dw + i);  // 52 MB per layer that nothing reads before the step ends
        }
    });
}

// Raise a kernel's dynamic-LDS limit: once per (device, kernel), remembered afterwards.
int set_lds_once(const void* kern, int bytes)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void*>, int> done;  // largest size already granted
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) dev = -1;
    std::lock_guard<std::mutex> lock(mu);
    int& have = done[std::make_pair(dev, kern)];
    if (dev >= 0 && have >= bytes) return W2L_OK;
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    have = bytes;
    return W2L_OK;
}
template <class K>
int set_lds(K kern, int bytes) { return set_lds_once((const void*)kern, bytes); }

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

// How to cut a tiles_m x tiles_n grid into 8 rectangular blocks, one per XCD: the cut (xm blocks along m,
// 8 / xm along n) that makes an L2 stream the fewest bytes, given the bytes one row of tiles (bytes_m) and one
// column of tiles (bytes_n) read.  0 if the grid does not divide.
int xcd_split(long long tiles_m, long long tiles_n, double bytes_m, double bytes_n)
{
    int best = 0;
    double best_cost = 0;
    for (int xm = 1; xm <= 8; xm *= 2) {
        const int xn = 8 / xm;
        if (tiles_m % xm || tiles_n % xn) continue;
        const double cost = (double)(tiles_m / xm) * bytes_m + (double)(tiles_n / xn) * bytes_n;
        if (!best || cost < best_cost) { best = xm; best_cost = cost; }
    }
    return best;
}

// The same for the split data gradient: 2 reduction halves x 4 blocks of tiles.  0 if the grid does not divide.
int xcd_split4(long long tiles_m, long long tiles_n, double bytes_m, double bytes_n)
{
    int best = 0;
    double best_cost = 0;
    for (int xm = 1; xm <= 4; xm *= 2) {
        const int xn = 4 / xm;
        if (tiles_m % xm || tiles_n % xn) continue;
        const double cost = (double)(tiles_m / xm) * bytes_m + (double)(tiles_n / xn) * bytes_n;
        if (!best || cost < best_cost) { best = xm; best_cost = cost; }
    }
    return best;
}

bool common_ok(const ConvDesc& d)
{
    if (d.Cin % 8 || d.Cout % 8) return false;
    if ((long long)d.k * d.Cin > 32767 * 8LL || (long long)d.k * d.Cout > 32767 * 8LL) return false;
    // 32-bit element/byte offsets inside the kernels
    if (((long long)d.B * d.x_pitch + d.slack) * d.Cin >= (1LL << 30)) return false;
    if (((long long)d.B * d.y_pitch + d.slack) * d.Cout >= (1LL << 30)) return false;
    if ((long long)d.Cout * d.k * d.Cin >= (1LL << 30)) return false;
    return true;
}
// FAST addressing: windows never leave zero-filled, allocated memory
bool halo_ok_x(const ConvDesc& d) { return d.p == 0 || d.x_halo >= d.p; }
bool halo_ok_y(const ConvDesc& d) { return d.p == 0 || d.y_halo >= d.p; }

// Activation-slab kernels: stride 1, the slab tensor has C % 64 == 0 channels and a halo, at
// least two taps, a slab of srows frames covers the tile's window, and the last tile's slab
// stays inside the allocation (B * pitch + slack frames).
bool slab_ok(const ConvDesc& d, int bm, int srows, int C, int frames, int pitch, int halo)
{
    if (d.s != 1 || d.k < 2 || C % 64 != 0 || halo < d.p || halo == 0 || bm + d.k - 1 > srows) return false;
    const long long F = (long long)(d.B - 1) * pitch + frames;
    const long long last_f0 = halo + (F - 1) / bm * bm;
    return last_f0 - d.p + srows <= (long long)d.B * pitch + d.slack;
}

// tile -> (panel depth, ring depth): 3 x 48 KB for the tiles that fit, 4 x 32 KB for 256x256
// and the groups of wavefronts: two reduction groups, or for 256x256 two column groups
#define W2L_TILE_DISPATCH(CALL)                                                \
    if (tc.bm == 256 && tc.bn == 256) { CALL(256, 256, 32, 4, 1, 2); }         \
    else if (tc.bm == 192 && tc.bn == 192) { CALL(192, 192, 64, 3, 2, 1); }    \
    else if (tc.bm == 256 && tc.bn == 128) { CALL(256, 128, 64, 3, 2, 1); }    \
    else if (tc.bm == 128 && tc.bn == 256) { CALL(128, 256, 64, 3, 2, 1); }    \
    else { CALL(128, 128, 64, 3, 2, 1); }

}  // namespace

bool conv_fwd_mfma_ok(const ConvDesc& d)
{
    // rows of w are fetched in 16-byte chunks along (j,ci): only Cin needs to be a multiple of 8
    ConvDesc e = d;
    e.Cout = (d.Cout + 7) / 8 * 8;
    return d.Cin % 8 == 0 && common_ok(e) && d.Cout >= 16 && (long long)d.B * d.Tp >= 128;
}

// XCD cut of the 192x192 slab forward's tile grid: a row of tiles reads its 192 + k - 1 frames of x, a column
// of tiles its 192 rows of w
static int fwd_slab_xcd(const ConvDesc& g, long long tiles_m, long long tiles_n)
{
    return xcd_split(tiles_m, tiles_n, (double)(192 + g.k - 1) * g.Cin, 192.0 * g.k * g.Cin);
}

int conv_fwd_mfma(const ConvDesc& g0, const void* x, const void* w, const float* bias, void* y, int ydt, hipStream_t st)
{
    ConvDesc g = g0;
    const long long M = (long long)g.B * g.Tp, N = g.Cout;
    const TileChoice tc = choose_tile(M, N);
    const bool fast = halo_ok_x(g) && ((long long)g.k * g.Cin) % 64 == 0;
    int rc = W2L_OK;
    if (fast && tc.bm == 192 && tc.bn == 192 && slab_ok(g, 192, 256, g.Cin, g.T, g.x_pitch, g.x_halo)) {
        constexpr int bytes = slab_lds_bytes(192, 192, 256, 2);
        const long long F = (long long)(g.B - 1) * g.x_pitch + g.T;
        const unsigned grid = (unsigned)(((F + 191) / 192) * ((N + 191) / 192));
        g.xcd_m = fwd_slab_xcd(g, (F + 191) / 192, (N + 191) / 192);
        if (ydt == W2L_BF16) {
            rc = set_lds(conv_fwd_slab_k<192, 192, 256, 2, bf16_t, false>, bytes);
            if (!rc) hipLaunchKernelGGL((conv_fwd_slab_k<192, 192, 256, 2, bf16_t, false>), dim3(grid), dim3(512), bytes, st, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)y, (bf16_t*)nullptr, g);
        } else {
            rc = set_lds(conv_fwd_slab_k<192, 192, 256, 2, float, false>, bytes);
            if (!rc) hipLaunchKernelGGL((conv_fwd_slab_k<192, 192, 256, 2, float, false>), dim3(grid), dim3(512), bytes, st, (const bf16_t*)x, (const bf16_t*)w, bias, (float*)y, (bf16_t*)nullptr, g);
        }
        return rc ? rc : launch_status();
    }
#define LAUNCH(KERN, BYTES, ...)                                                          \
    {                                                                                     \
        rc = set_lds(KERN, BYTES);                                                        \
        if (!rc) hipLaunchKernelGGL(KERN, dim3(grid), dim3(nthreads), BYTES, st, __VA_ARGS__);  \
    }
#define CALL(BM_, BN_, BK_, ST_, KG_, GN_)                                                                         \
    {                                                                                                         \
        constexpr int bytes = ST_ * (BM_ + BN_) * BK_ * 2;                                                    \
        const unsigned nthreads = 256 * KG_ * GN_;                                                                  \
        const unsigned grid = (unsigned)(((M + BM_ - 1) / BM_) * ((N + BN_ - 1) / BN_));                      \
        if (ydt == W2L_BF16) {                                                                                \
            if (fast) LAUNCH((conv_fwd_k<BM_, BN_, BK_, ST_, KG_, GN_, true, bf16_t>), bytes, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)y, g) \
            else LAUNCH((conv_fwd_k<BM_, BN_, BK_, ST_, KG_, GN_, false, bf16_t>), bytes, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)y, g)     \
        } else {                                                                                              \
            if (fast) LAUNCH((conv_fwd_k<BM_, BN_, BK_, ST_, KG_, GN_, true, float>), bytes, (const bf16_t*)x, (const bf16_t*)w, bias, (float*)y, g)   \
            else LAUNCH((conv_fwd_k<BM_, BN_, BK_, ST_, KG_, GN_, false, float>), bytes, (const bf16_t*)x, (const bf16_t*)w, bias, (float*)y, g)       \
        }                                                                                                     \
    }
    W2L_TILE_DISPATCH(CALL)
#undef CALL
    return rc ? rc : launch_status();
}

bool conv_fwd_glu_ok(const ConvDesc& d)
{
    // the 192x192 slab kernel with the two GLU halves interleaved per tile; h in the time layout of x
    const long long M = (long long)d.B * d.Tp;
    const TileChoice tc = choose_tile(M, d.Cout);
    return conv_fwd_mfma_ok(d) && halo_ok_x(d) && tc.bm == 192 && tc.bn == 192 && d.Cout % 2 == 0 && (d.Cout / 2) % 96 == 0 &&
           d.T == d.Tp && d.slack >= LAYOUT_SLACK_ZERO && slab_ok(d, 192, 256, d.Cin, d.T, d.x_pitch, d.x_halo);
}

int conv_fwd_glu(const ConvDesc& g0, const void* x, const void* w, const float* bias, void* y, void* h, hipStream_t st)
{
    if (!conv_fwd_glu_ok(g0)) return W2L_ERR_SHAPE;
    ConvDesc g = g0;
    constexpr int bytes = slab_lds_bytes(192, 192, 256, 2);
    const long long F = (long long)(g.B - 1) * g.x_pitch + g.T;
    const unsigned grid = (unsigned)(((F + 191) / 192) * (g.Cout / 192));
    g.xcd_m = fwd_slab_xcd(g, (F + 191) / 192, g.Cout / 192);
    int rc = set_lds(conv_fwd_slab_k<192, 192, 256, 2, bf16_t, true>, bytes);
    if (!rc) hipLaunchKernelGGL((conv_fwd_slab_k<192, 192, 256, 2, bf16_t, true>), dim3(grid), dim3(512), bytes, st, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)y, (bf16_t*)h, g);
    return rc ? rc : launch_status();
}

bool conv_dgrad_mfma_ok(const ConvDesc& d)
{
    return d.s == 1 && common_ok(d) && d.Cout % 64 == 0 && d.Cin >= 64 && (long long)d.B * d.T >= 128;
}

// Split-reduction data gradient: 192x192 tiles, two workgroups per tile that each reduce half of the
// channel blocks; the second of a pair to finish adds the first one's fp32 sums (left in scratch) and
// writes the tile.  Taken when one workgroup per tile would leave more than a third of the CUs idle
// and two per tile fit the chip in one round.
// Scratch: DGRAD_TICKET_BYTES of tickets (one int per tile), then two fp32 slots of 192 x 192 per tile.
bool dgrad_split_ok(const ConvDesc& g)
{
    if (!conv_dgrad_mfma_ok(g) || !halo_ok_y(g) || g.Cin % 8 != 0 || (g.Cout / 64) % 2 != 0 || g.Cout < 256) return false;
    if (!slab_ok(g, 192, 256, g.Cout, g.Tp, g.y_pitch, g.y_halo)) return false;
    const long long M = (long long)g.B * g.T, N = g.Cin, F = (long long)(g.B - 1) * g.y_pitch + g.Tp;
    const TileChoice tc = choose_tile(M, N);
    const long long t1 = ((M + tc.bm - 1) / tc.bm) * ((N + tc.bn - 1) / tc.bn);
    const long long t2 = ((F + 191) / 192) * ((N + 191) / 192);
    return t1 <= 170 && 2 * t2 <= 256 && 2 * t2 > t1;
}
size_t conv_dgrad_scratch_bytes(const ConvDesc& g)
{
    if (!dgrad_split_ok(g)) return 0;
    const long long F = (long long)(g.B - 1) * g.y_pitch + g.Tp;
    const size_t tiles = (size_t)((F + 191) / 192) * ((g.Cin + 191) / 192);
    return DGRAD_TICKET_BYTES + tiles * 2 * 192 * 192 * 4;
}

// grid and XCD cut of the split data gradient's launch (two workgroups per 192x192 tile)
static dim3 dgrad_split_grid(ConvDesc& g, long long tiles_m, long long tiles_n)
{
    g.xcd_m = xcd_split4(tiles_m, tiles_n, (double)(192 + g.k - 1) * g.Cout / 2, 192.0 * g.k * g.Cout / 2);
    const unsigned tiles = (unsigned)(tiles_m * tiles_n);
    return g.xcd_m > 0 ? dim3(2 * tiles) : dim3(tiles, 2);
}

int conv_dgrad_mfma(const ConvDesc& g0, const void* dy, const void* w, void* dx, void* scratch, size_t scratch_bytes,
                    hipStream_t st, bool tickets_zeroed)
{
    ConvDesc g = g0;
    const long long M = (long long)g.B * g.T, N = g.Cin;
    const TileChoice tc = choose_tile(M, N);
    const bool fast = halo_ok_y(g);
    int rc = W2L_OK;
    if (scratch && dgrad_split_ok(g) && scratch_bytes >= conv_dgrad_scratch_bytes(g)) {
        constexpr int bytes = slab_lds_bytes(192, 192, 256, 2);
        const long long F = (long long)(g.B - 1) * g.y_pitch + g.Tp;
        const int tiles = (int)(((F + 191) / 192) * ((N + 191) / 192));
        int* tickets = static_cast<int*>(scratch);
        float* part = reinterpret_cast<float*>(static_cast<unsigned char*>(scratch) + DGRAD_TICKET_BYTES);
        if (!tickets_zeroed) {
            hipLaunchKernelGGL(zero_rows_k, dim3(1), dim3(256), 0, st, (bf16_t*)nullptr, 0LL, 0LL, 0LL, 0LL, 8, tickets, tiles);
            rc = launch_status();
            if (rc) return rc;
        }
        rc = set_lds(conv_dgrad_slab_k<192, 192, 256, 2, false>, bytes);
        if (rc) return rc;
        const dim3 grid = dgrad_split_grid(g, (F + 191) / 192, (N + 191) / 192);
        hipLaunchKernelGGL((conv_dgrad_slab_k<192, 192, 256, 2, false>), grid, dim3(512), bytes, st, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, (const bf16_t*)nullptr, part, tickets, g);
        g.xcd_m = 0;
        return launch_status();
    }
    if (fast && tc.bm == 256 && tc.bn == 128 && slab_ok(g, 256, 320, g.Cout, g.Tp, g.y_pitch, g.y_halo)) {
        constexpr int bytes = slab_lds_bytes(256, 128, 320, 2);
        const long long F = (long long)(g.B - 1) * g.y_pitch + g.Tp;
        const unsigned grid = (unsigned)(((F + 255) / 256) * ((N + 127) / 128));
        rc = set_lds(conv_dgrad_slab_k<256, 128, 320, 2, false>, bytes);
        if (!rc) hipLaunchKernelGGL((conv_dgrad_slab_k<256, 128, 320, 2, false>), dim3(grid), dim3(512), bytes, st, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, (const bf16_t*)nullptr, (float*)nullptr, (int*)nullptr, g);
        return rc ? rc : launch_status();
    }
#define CALL(BM_, BN_, BK_, ST_, KG_, GN_)                                                                     \
    {                                                                                                     \
        constexpr int bytes = ST_ * (BM_ + BN_) * BK_ * 2;                                                \
        const unsigned nthreads = 256 * KG_ * GN_;                                                              \
        const unsigned grid = (unsigned)(((M + BM_ - 1) / BM_) * ((N + BN_ - 1) / BN_));                  \
        if (fast) LAUNCH((conv_dgrad_k<BM_, BN_, BK_, ST_, KG_, GN_, true>), bytes, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, g) \
        else LAUNCH((conv_dgrad_k<BM_, BN_, BK_, ST_, KG_, GN_, false>), bytes, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, g)     \
    }
    W2L_TILE_DISPATCH(CALL)
#undef CALL
    return rc ? rc : launch_status();
}

bool conv_dgrad_glu_ok(const ConvDesc& d)
{
    // the slab kernel's tile, dy haloed, and dy of the layer below in the same time layout
    return conv_dgrad_mfma_ok(d) && halo_ok_y(d) && d.Cin % 8 == 0 && d.x_pitch == d.y_pitch && d.x_halo == d.y_halo &&
           d.T == d.Tp && d.slack >= LAYOUT_SLACK_ZERO && slab_ok(d, 256, 320, d.Cout, d.Tp, d.y_pitch, d.y_halo);
}

int conv_dgrad_glu(const ConvDesc& g0, const void* dy, const void* w, const void* yprev, void* dyprev, void* scratch,
                   size_t scratch_bytes, hipStream_t st)
{
    if (!conv_dgrad_glu_ok(g0)) return W2L_ERR_SHAPE;
    ConvDesc g = g0;
    const long long F = (long long)(g.B - 1) * g.y_pitch + g.Tp;
    const long long z_end = (long long)g.B * g.y_pitch + LAYOUT_SLACK_ZERO;
    if (scratch && dgrad_split_ok(g) && scratch_bytes >= conv_dgrad_scratch_bytes(g)) {
        // two workgroups per 192x192 tile; the one that finishes a tile applies the GLU backward in its epilogue
        constexpr int bytes = slab_lds_bytes(192, 192, 256, 2);
        const long long tiles_m = (F + 191) / 192;
        const int tiles = (int)(tiles_m * ((g.Cin + 191) / 192));
        int* tickets = static_cast<int*>(scratch);
        float* part = reinterpret_cast<float*>(static_cast<unsigned char*>(scratch) + DGRAD_TICKET_BYTES);
        // frames the tiles do not cover (leading halo; end of the last tile to the end of the zeroed slack), and the tickets
        const long long t_end = g.y_halo + tiles_m * 192;
        hipLaunchKernelGGL(zero_rows_k, dim3(64), dim3(256), 0, st, (bf16_t*)dyprev, 0LL, (long long)g.y_halo, t_end,
                           t_end > z_end ? t_end : z_end, 2 * g.Cin, tickets, tiles);
        int rc = launch_status();
        if (rc) return rc;
        rc = set_lds(conv_dgrad_slab_k<192, 192, 256, 2, true>, bytes);
        if (rc) return rc;
        const dim3 grid = dgrad_split_grid(g, tiles_m, (g.Cin + 191) / 192);
        hipLaunchKernelGGL((conv_dgrad_slab_k<192, 192, 256, 2, true>), grid, dim3(512), bytes, st, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dyprev, (const bf16_t*)yprev, part, tickets, g);
        return launch_status();
    }
    constexpr int BM = 256, BN = 128;
    constexpr int bytes = slab_lds_bytes(BM, BN, 320, 2);
    const long long tiles_m = (F + BM - 1) / BM;
    // frames the tiles do not cover: the leading halo, and from the end of the last tile to the end of the zeroed slack
    const long long t_end = g.y_halo + tiles_m * BM;
    hipLaunchKernelGGL(zero_rows_k, dim3(64), dim3(256), 0, st, (bf16_t*)dyprev, 0LL, (long long)g.y_halo, t_end,
                       t_end > z_end ? t_end : z_end, 2 * g.Cin, (int*)nullptr, 0);
    int rc = launch_status();
    if (rc) return rc;
    const unsigned grid = (unsigned)(tiles_m * ((g.Cin + BN - 1) / BN));
    rc = set_lds(conv_dgrad_slab_k<BM, BN, 320, 2, true>, bytes);
    if (!rc) hipLaunchKernelGGL((conv_dgrad_slab_k<BM, BN, 320, 2, true>), dim3(grid), dim3(512), bytes, st, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dyprev, (const bf16_t*)yprev, (float*)nullptr, (int*)nullptr, g);
    return rc ? rc : launch_status();
}

bool conv_wgrad_mfma_ok(const ConvDesc& d)
{
    return common_ok(d) && d.Cout >= 64 && (long long)d.k * d.Cin >= 64;
}

// FAST walks the frames of both tensors in lock step and over-reads up to 64 + p frames
static bool wgrad_fast(const ConvDesc& g)
{
    return g.s == 1 && g.x_pitch == g.y_pitch && g.x_halo == g.y_halo && g.x_halo >= g.p && g.slack >= 64 &&
           (g.B == 1 || g.x_halo > 0 || g.p == 0);
}

bool conv_wgrad_mfma_takes_dbias(const ConvDesc& d) { return conv_wgrad_mfma_ok(d) && wgrad_fast(d); }

int conv_wgrad_mfma(const ConvDesc& g, const void* x, const void* dy, float* dw, float* dbias, int accumulate, hipStream_t st)
{
    const long long M = g.Cout, N = g.w_cols ? g.w_cols : (long long)g.k * g.Cin;
    const TileChoice tc = choose_tile(M, N);
    const bool fast = wgrad_fast(g);
    if (g.w_cols && !fast) return W2L_ERR_SHAPE;  // a folded layer exists only in the dense walk through the frames
    if (dbias && !fast) return W2L_ERR_SHAPE;  // callers ask conv_wgrad_mfma_takes_dbias() first
    const long long extra = dbias ? 1 : 0;     // the column of tiles that yields the bias gradient
    int rc = W2L_OK;
#define CALL(BM_, BN_, BK_, ST_, KG_, GN_)                                                                     \
    {                                                                                                     \
        constexpr int bytes = ST_ * (BM_ + BN_) * BK_ * 2;                                                \
        const unsigned nthreads = 256 * KG_ * GN_;                                                              \
        const unsigned grid = (unsigned)(((M + BM_ - 1) / BM_) * ((N + BN_ - 1) / BN_ + extra));          \
        if (fast && dbias) LAUNCH((conv_wgrad_k<BM_, BN_, BK_, ST_, KG_, GN_, true, true>), bytes, (const bf16_t*)x, (const bf16_t*)dy, dw, dbias, g, accumulate) \
        else if (fast) LAUNCH((conv_wgrad_k<BM_, BN_, BK_, ST_, KG_, GN_, true, false>), bytes, (const bf16_t*)x, (const bf16_t*)dy, dw, (float*)nullptr, g, accumulate) \
        else LAUNCH((conv_wgrad_k<BM_, BN_, BK_, ST_, KG_, GN_, false, false>), bytes, (const bf16_t*)x, (const bf16_t*)dy, dw, (float*)nullptr, g, accumulate) \
    }
    W2L_TILE_DISPATCH(CALL)
#undef CALL
#undef LAUNCH
    return rc ? rc : launch_status();
}

}  // namespace w2l
