// Internal helpers of libw2l (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/w2l.h"

namespace w2l {

typedef unsigned short bf16_t;  // raw bits: upper half of an IEEE float

void note_hip_error(hipError_t e);
// status of the launch just made on this thread
inline int launch_status() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    return W2L_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int out_len(int T, int s) { return (T + s - 1) / s; }
inline size_t dtype_size(int dt) { return dt == W2L_BF16 ? 2 : 4; }
inline bool valid_dtype(int dt) { return dt == W2L_F32 || dt == W2L_BF16; }

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
// round to nearest, ties to even; NaN stays NaN.  gfx950 converts in hardware (v_cvt_pk_bf16_f32, which the
// compiler selects for this cast and pairs up for neighbouring values): one instruction instead of six.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

// the hardware reciprocal (1 ulp) instead of an IEEE division: a quarter of the GLU kernels' instructions
__device__ __forceinline__ float sigmoidf_(float u) { return __builtin_amdgcn_rcpf(1.f + __expf(-u)); }

// Time layout of the activations the library keeps itself (train step workspace, staged
// operands of the convolution entry points): LAYOUT_HALO zero frames on both sides of every
// utterance, then LAYOUT_SLACK allocated frames after the last utterance, of which the first
// LAYOUT_SLACK_ZERO are kept zero (kernels whose reduction runs through the frames over-read
// into them); the rest is only ever read for outputs that are dropped.
constexpr int LAYOUT_HALO = 8, LAYOUT_SLACK = 320, LAYOUT_SLACK_ZERO = 64;

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p, size_t i) { return p[i]; }
    static __device__ __forceinline__ void store(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
    static __device__ __forceinline__ void store(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }
};

// ---- internal entry points shared between translation units -----------------------
// Geometry of one convolution plus the memory layout of the time axis of its tensors.
// Utterance b, frame t of the input-side tensor (x, dx) lives at element
// ((b * x_pitch + x_halo + t) * Cin); of the output-side tensor (y, dy) at
// ((b * y_pitch + y_halo + t') * Cout).  A tensor with halo > 0 holds zeros in frames
// [-halo, 0) and [T, pitch - halo) of every utterance, and `slack` further zero frames
// after its last utterance; tensor pointers always point at the start of the allocation
// (frame -halo of utterance 0).  Caller-supplied (C ABI) tensors are dense: pitch = T,
// halo = 0, slack = 0.
struct ConvDesc {
    int B, T, Tp, Cin, Cout, k, s, p;
    int x_pitch, x_halo, y_pitch, y_halo, slack;
    int xcd_m = 0;  // set by the launchers: how the tile grid is cut over the 8 XCDs (see tile_of_block)
    int w_cols = 0; // weight gradient only: columns of a dw row that exist (0: all k * Cin).  A strided layer
                    // folded into a stride-1 one (fold_stride) has k * Cin rounded up to whole folded frames.
};
inline ConvDesc dense_desc(int B, int T, int Cin, int Cout, int k, int s)
{
    ConvDesc d{B, T, out_len(T, s), Cin, Cout, k, s, (k - 1) / 2, 0, 0, 0, 0, 0, 0, 0};
    d.x_pitch = T;
    d.y_pitch = d.Tp;
    return d;
}

// A layer with stride s > 1 read as a stride-1 layer over frames folded s at a time: x[B,T,Cin] is, as it lies
// in memory, also [B, T/s, s*Cin], and the window of output frame t' -- frames s t' - p .. s t' - p + k - 1 -- is
// the folded frames t' - p/s .. of a kernel of width ceil(k/s) whose weight rows are the same memory, k * Cin long
// (the folded kernel's last, partial tap has no weights: w_cols marks where a row ends).  Needs p % s == 0 and
// T % s == 0.  Used for the weight gradient of the strided first layer, whose reduction then runs densely through
// the frames like every other layer's.  Returns false if the layer does not fold.
inline bool fold_stride(const ConvDesc& d, ConvDesc& f)
{
    if (d.s <= 1 || d.p % d.s != 0 || d.T % d.s != 0 || d.x_pitch % d.s != 0 || d.x_halo % d.s != 0) return false;
    f = d;
    f.T = f.Tp = d.T / d.s;
    f.x_pitch = d.x_pitch / d.s;  // the time layout of x in folded frames
    f.x_halo = d.x_halo / d.s;
    f.Cin = d.Cin * d.s;
    f.k = 2 * (d.p / d.s) + 1;               // symmetric: (k - 1) / 2 = p / s frames either side
    if ((long long)f.k * f.Cin < (long long)d.k * d.Cin) return false;
    f.s = 1;
    f.p = d.p / d.s;
    f.w_cols = d.k * d.Cin;
    return true;
}

// dispatchers (api.hip): MFMA kernels where the shape allows, shape-agnostic kernels otherwise
int conv_fwd(const ConvDesc& d, const void* x, const void* w, const float* bias, void* y, int dt, int ydt,
             hipStream_t st);
// scratch (optional): conv_dgrad_scratch_bytes(d) bytes of device memory; given it, shapes that would
// leave CUs idle split their reduction over two workgroups per tile
int conv_dgrad(const ConvDesc& d, const void* dy, const void* w, void* dx, int dt, int dydt, hipStream_t st,
               void* scratch = nullptr, size_t scratch_bytes = 0);
size_t conv_dgrad_scratch_bytes(const ConvDesc& d);
// scratch: conv_wgrad_scratch_bytes() bytes of device memory
size_t conv_wgrad_scratch_bytes(int Cin, int Cout, int k);
// true where conv_wgrad() produces dbias inside the weight-gradient launch (no separate column-sum kernels)
bool conv_wgrad_fuses_dbias(const ConvDesc& d, int dt, int dydt);
int conv_wgrad(const ConvDesc& d, const void* x, const void* dy, float* dw, float* dbias, int dt, int dydt,
               int accumulate, void* scratch, hipStream_t st);

int conv_fwd_generic(const ConvDesc& d, const void* x, const void* w, const float* bias, void* y, int dt, int ydt,
                     hipStream_t st);
int conv_dgrad_generic(const ConvDesc& d, const void* dy, const void* w, void* dx, int dt, int dydt, hipStream_t st);
int conv_wgrad_generic(const ConvDesc& d, const void* x, const void* dy, float* dw, int dt, int dydt, int accumulate,
                       hipStream_t st);
// narrow outputs (Cout <= 32): row-chunked reduction, SKINNY_CHUNKS partials summed in a fixed order
enum { SKINNY_CHUNKS = 64 };
size_t conv_wgrad_skinny_scratch(int Cin, int Cout, int k);
int conv_wgrad_skinny(const ConvDesc& d, const void* x, const void* dy, float* dw, int dt, int dydt, int accumulate,
                      float* scratch, hipStream_t st);
// column sums of dy[rows,Cout] -> dbias, two deterministic stages; scratch holds DBIAS_CHUNKS*Cout floats
enum { DBIAS_CHUNKS = 64 };
int dbias_reduce(const void* dy, float* dbias, long long rows, int Cout, int dydt, int accumulate,
                 float* scratch, hipStream_t st);

// MFMA (bf16 operands, fp32 accumulate) paths; *_ok() says whether a shape is taken
bool conv_fwd_mfma_ok(const ConvDesc& d);
int conv_fwd_mfma(const ConvDesc& d, const void* x, const void* w, const float* bias, void* y, int ydt, hipStream_t st);
bool conv_dgrad_mfma_ok(const ConvDesc& d);
// tickets_zeroed: the first DGRAD_TICKET_BYTES of scratch are already zero on the stream (the caller's staging
// launch cleared them), so the launch that would clear them is left out
int conv_dgrad_mfma(const ConvDesc& d, const void* dy, const void* w, void* dx, void* scratch, size_t scratch_bytes,
                    hipStream_t st, bool tickets_zeroed = false);
constexpr size_t DGRAD_TICKET_BYTES = 1024;
// forward pass fused with the layer's GLU: writes y (dense, pre-GLU, bf16) and h = GLU(y) into a
// haloed tensor with the time layout of x (halo frames and the zeroed slack written as zeros)
bool conv_fwd_glu_ok(const ConvDesc& d);
int conv_fwd_glu(const ConvDesc& d, const void* x, const void* w, const float* bias, void* y, void* h, hipStream_t st);
// data gradient of a layer fused with the GLU backward of the layer below it: instead of dx (=
// dh of the layer below) it writes dy of the layer below, dy = GLU'(yprev) * dh, into a haloed
// tensor with the same time layout as this layer's dy (halo frames are written as zeros).
// yprev: dense [B*T, 2*Cin] pre-GLU activations of the layer below.
bool conv_dgrad_glu_ok(const ConvDesc& d);
// scratch (optional): conv_dgrad_scratch_bytes(d) bytes; given it, shapes dgrad_split_ok(d) accepts take
// the split-reduction tiles and the GLU backward moves into their combining pass
int conv_dgrad_glu(const ConvDesc& d, const void* dy, const void* w, const void* yprev, void* dyprev, void* scratch,
                   size_t scratch_bytes, hipStream_t st);
bool dgrad_split_ok(const ConvDesc& d);
bool conv_wgrad_mfma_ok(const ConvDesc& d);
// dbias (nullable): only where conv_wgrad_mfma_takes_dbias(d) -- the bias gradient comes out of the same launch
bool conv_wgrad_mfma_takes_dbias(const ConvDesc& d);
int conv_wgrad_mfma(const ConvDesc& d, const void* x, const void* dy, float* dw, float* dbias, int accumulate, hipStream_t st);

// w2l_ctc_fwd_bwd with in_len counted before a total stride len_div (ctc.hip): the criterion sees ceil(in_len / len_div)
int ctc_fwd_bwd_strided(const float* input, int is_logits, const int* targets, const int* in_len, const int* tgt_len,
                        float* loss, float* grad, int B, int Tp, int C, int Lmax, int blank, float grad_scale,
                        void* workspace, size_t ws_bytes, void* stream, int len_div);

// GLU with an explicit output layout (elementwise.hip).  y (and dh) are dense [B*Tp, Cout]
// ([B*Tp, Cout/2]); the output is written with the given pitch and halo, halo and slack
// frames included (as zeros).
int glu_fwd_layout(const void* y, void* h, int B, int Tp, int Cout, int dtype, int pitch, int halo, int slack,
                   hipStream_t st);
int glu_bwd_layout(const void* y, const void* dh, void* dy, int B, int Tp, int Cout, int dtype, int pitch, int halo,
                   int slack, hipStream_t st);

// dense bf16 [B*Tp, C] (C % 8 == 0) -> layout with the given pitch / halo / slack, zeros outside the real frames
// (and `nclear` integers at `clear` set to zero on the way)
int pad_layout_bf16(const void* src, void* dst, int B, int Tp, int C, int pitch, int halo, int slack, hipStream_t st,
                    int* clear = nullptr, int nclear = 0);
// any dtype, any channel count
int pad_layout(const void* src, void* dst, int B, int Tp, int C, int dtype, int pitch, int halo, int slack, hipStream_t st);
// data-gradient operand preparation (elementwise.hip): dy (fp32 or bf16, dense [B*Tp, C]) -> bf16 in the haloed layout
// with the channels padded by zeros to Cp; w[Cout][k][Cin] -> [Cp][kf][s*Cin] with the stride folded into the
// channels (w'[co][jj][ph*Cin+ci] = w[co][s*jj+ph][ci]) and zeros for taps and rows that do not exist
int prep_dgrad_dy(const void* src, int src_dtype, void* dst, int B, int Tp, int C, int Cp, int pitch, int halo, int slack,
                  hipStream_t st, int* clear = nullptr, int nclear = 0);
int prep_dgrad_w(const void* w, void* dst, int Cout, int k, int Cin, int Cp, int kf, int s, hipStream_t st);
// A data gradient brought into the form the MFMA kernels take (api.hip).  ok: the shape can be prepared; d: the
// geometry of the prepared problem (stride 1, Cout a multiple of 64, dy haloed); copy_w: the weights need the
// padded / folded copy.  Workspace: dy_bytes, then w_bytes, then split_bytes (conv_dgrad_scratch_bytes(d)).
struct DgradPrep {
    bool ok = false, copy_w = false;
    ConvDesc d;
    int Cout = 0, k = 0, Cin = 0, s = 1;  // the layer as the caller describes it
    size_t dy_bytes = 0, w_bytes = 0, split_bytes = 0;
    size_t total() const { return dy_bytes + w_bytes + split_bytes; }
};
DgradPrep dgrad_prep(int B, int T, int Cin, int Cout, int k, int s, int dt);
// dy: dense [B, Tp, Cout] of dtype dydt; dx: dense [B, T, Cin] bf16; ws: prep.total() bytes, 256-byte aligned
int conv_dgrad_prepared(const DgradPrep& prep, const void* dy, int dydt, const void* w, void* dx, void* ws, hipStream_t st);
// the same for two tensors that share B, Tp and the layout, in one launch
int pad_layout2_bf16(const void* src0, void* dst0, int C0, const void* src1, void* dst1, int C1, int B, int Tp, int pitch,
                     int halo, int slack, hipStream_t st);

}  // namespace w2l
