// C-ABI entry points for the temporal convolution and the library's bookkeeping calls.
// Argument checks happen here, on the host, before any launch; the kernels assume
// the shapes they are given.
#include "common.h"

namespace w2l {
static thread_local int g_last_hip_error = 0;
void note_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace w2l

using namespace w2l;

extern "C" int w2l_version(void) { return 100; }

extern "C" int w2l_last_hip_error(void) { return g_last_hip_error; }

extern "C" const char* w2l_status_str(int s)
{
    switch (s) {
        case W2L_OK: return "ok";
        case W2L_ERR_NULL: return "null pointer";
        case W2L_ERR_SHAPE: return "bad shape";
        case W2L_ERR_DTYPE: return "bad dtype";
        case W2L_ERR_ALIGN: return "pointer not 16-byte aligned";
        case W2L_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case W2L_ERR_TARGET: return "bad target label or length";
        case W2L_ERR_LAUNCH: return "HIP launch failed";
        default: return "unknown status";
    }
}

namespace {
int check_conv_shape(int B, int T, int Cin, int Cout, int k, int s)
{
    if (B <= 0 || T <= 0 || Cin <= 0 || Cout <= 0 || k <= 0 || s <= 0) return W2L_ERR_SHAPE;
    if ((k & 1) == 0) return W2L_ERR_SHAPE;
    if ((long long)B * T > (1LL << 30) || (long long)k * Cin > (1LL << 30) || (long long)k * Cout > (1LL << 30))
        return W2L_ERR_SHAPE;
    return W2L_OK;
}
bool ws_ok(void* ws, size_t have, size_t need)
{
    if (need == 0) return true;
    return ws && have >= need && (reinterpret_cast<uintptr_t>(ws) & 255u) == 0;
}
}  // namespace

namespace w2l {

int conv_fwd(const ConvDesc& d, const void* x, const void* w, const float* bias, void* y, int dt, int ydt,
             hipStream_t st)
{
    if (dt == W2L_BF16 && conv_fwd_mfma_ok(d)) return conv_fwd_mfma(d, x, w, bias, y, ydt, st);
    return conv_fwd_generic(d, x, w, bias, y, dt, ydt, st);
}

int conv_dgrad(const ConvDesc& d, const void* dy, const void* w, void* dx, int dt, int dydt, hipStream_t st,
               void* scratch, size_t scratch_bytes)
{
    if (dt == W2L_BF16 && dydt == W2L_BF16 && conv_dgrad_mfma_ok(d))
        return conv_dgrad_mfma(d, dy, w, dx, scratch, scratch_bytes, st);
    return conv_dgrad_generic(d, dy, w, dx, dt, dydt, st);
}

size_t conv_wgrad_scratch_bytes(int Cin, int Cout, int k)
{
    return round_up((size_t)DBIAS_CHUNKS * Cout * 4, 256) + conv_wgrad_skinny_scratch(Cin, Cout, k);
}

bool conv_wgrad_fuses_dbias(const ConvDesc& d, int dt, int dydt)
{
    return d.Cout > 32 && dt == W2L_BF16 && dydt == W2L_BF16 && conv_wgrad_mfma_takes_dbias(d);
}

int conv_wgrad(const ConvDesc& d, const void* x, const void* dy, float* dw, float* dbias, int dt, int dydt,
               int accumulate, void* scratch, hipStream_t st)
{
    float* dbias_scratch = static_cast<float*>(scratch);
    float* skinny_scratch =
        reinterpret_cast<float*>(static_cast<unsigned char*>(scratch) + round_up((size_t)DBIAS_CHUNKS * d.Cout * 4, 256));
    if (dbias && conv_wgrad_fuses_dbias(d, dt, dydt)) return conv_wgrad_mfma(d, x, dy, dw, dbias, accumulate, st);
    if (dbias) {
        // halo frames hold zeros, so summing every frame of the allocation is the same sum
        const int rc = dbias_reduce(dy, dbias, (long long)d.B * d.y_pitch, d.Cout, dydt, accumulate, dbias_scratch, st);
        if (rc) return rc;
    }
    if (d.Cout <= 32) return conv_wgrad_skinny(d, x, dy, dw, dt, dydt, accumulate, skinny_scratch, st);
    if (dt == W2L_BF16 && dydt == W2L_BF16 && conv_wgrad_mfma_ok(d)) return conv_wgrad_mfma(d, x, dy, dw, nullptr, accumulate, st);
    return conv_wgrad_generic(d, x, dy, dw, dt, dydt, accumulate, st);
}

}  // namespace w2l

namespace {
// The C ABI takes dense tensors; the MFMA kernels run fastest on tensors with a zero halo
// around every utterance.  Given workspace, the entry points first copy the window-read
// operand(s) into that layout (one bandwidth-bound pass, a few percent of the GEMM).
constexpr int ABI_HALO = LAYOUT_HALO, ABI_SLACK = LAYOUT_SLACK, ABI_SLACK_ZERO = LAYOUT_SLACK_ZERO;
size_t haloed_bytes(int B, int frames, int C) { return round_up(((size_t)B * (frames + 2 * ABI_HALO) + ABI_SLACK) * C * 2, 256); }
bool stage_fwd(int Cin, int Cout, int k, int s, int dt) { return dt == W2L_BF16 && k > 1 && (k - 1) / 2 <= ABI_HALO && Cin % 64 == 0 && Cout >= 16 && s >= 1; }
bool stage_wgrad(int Cin, int Cout, int k, int s, int dt) { return dt == W2L_BF16 && s == 1 && (k - 1) / 2 <= ABI_HALO && Cin % 8 == 0 && Cout % 8 == 0 && Cout >= 64 && (long long)k * Cin >= 64; }
// a strided layer whose stride folds into the channels (fold_stride) is staged as the stride-1 layer it folds to
bool stage_wgrad_folded(int B, int T, int Cin, int Cout, int k, int s, int dt, ConvDesc& f)
{
    return s > 1 && fold_stride(dense_desc(B, T, Cin, Cout, k, s), f) && stage_wgrad(f.Cin, Cout, f.k, 1, dt);
}
}  // namespace

extern "C" size_t w2l_conv1d_fwd_workspace_bytes(int B, int T, int Cin, int Cout, int k, int stride, int dtype)
{
    if (check_conv_shape(B, T, Cin, Cout, k, stride)) return 0;
    return stage_fwd(Cin, Cout, k, stride, dtype) ? haloed_bytes(B, T, Cin) : 0;
}

extern "C" int w2l_conv1d_fwd(const void* x, const void* w, const float* bias, void* y, int B, int T, int Cin,
                              int Cout, int k, int stride, int dtype, int y_dtype, void* workspace,
                              size_t ws_bytes, void* stream)
{
    if (!x || !w || !y) return W2L_ERR_NULL;
    int rc = check_conv_shape(B, T, Cin, Cout, k, stride);
    if (rc) return rc;
    if (!valid_dtype(dtype) || !valid_dtype(y_dtype) || (dtype == W2L_F32 && y_dtype != W2L_F32))
        return W2L_ERR_DTYPE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || (bias && !aligned16(bias))) return W2L_ERR_ALIGN;
    const size_t need = w2l_conv1d_fwd_workspace_bytes(B, T, Cin, Cout, k, stride, dtype);
    if (workspace && !ws_ok(workspace, ws_bytes, need)) return W2L_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    ConvDesc d = dense_desc(B, T, Cin, Cout, k, stride);
    if (workspace && need) {
        rc = pad_layout_bf16(x, workspace, B, T, Cin, T + 2 * ABI_HALO, ABI_HALO, ABI_SLACK_ZERO, st);
        if (rc) return rc;
        d.x_pitch = T + 2 * ABI_HALO;
        d.x_halo = ABI_HALO;
        d.slack = ABI_SLACK;
        x = workspace;
    }
    return conv_fwd(d, x, w, bias, y, dtype, y_dtype, st);
}

namespace w2l {
DgradPrep dgrad_prep(int B, int T, int Cin, int Cout, int k, int s, int dt)
{
    DgradPrep p;
    p.Cout = Cout; p.k = k; p.Cin = Cin; p.s = s;
    if (dt != W2L_BF16) return p;
    ConvDesc f = dense_desc(B, T, Cin, Cout, k, s);
    if (s > 1 && !fold_stride(dense_desc(B, T, Cin, Cout, k, s), f)) return p;   // a stride that does not fold
    f.w_cols = 0;
    const int Cp = (Cout + 63) / 64 * 64;
    p.copy_w = s > 1 || Cp != Cout;
    f.Cout = Cp;
    if (f.p > ABI_HALO) return p;
    f.y_pitch = f.Tp + 2 * ABI_HALO;
    f.y_halo = ABI_HALO;
    f.slack = ABI_SLACK;
    if (!conv_dgrad_mfma_ok(f)) return p;
    p.ok = true;
    p.d = f;
    p.dy_bytes = haloed_bytes(B, f.Tp, Cp);
    p.w_bytes = p.copy_w ? round_up((size_t)Cp * f.k * f.Cin * 2, 256) : 0;
    p.split_bytes = round_up(conv_dgrad_scratch_bytes(f), 256);
    return p;
}

int conv_dgrad_prepared(const DgradPrep& prep, const void* dy, int dydt, const void* w, void* dx, void* ws, hipStream_t st)
{
    if (!prep.ok) return W2L_ERR_SHAPE;
    const ConvDesc& f = prep.d;
    unsigned char* base = static_cast<unsigned char*>(ws);
    // the staging launch also zeroes the split reduction's tickets (the head of its scratch)
    int* const tickets = prep.split_bytes ? reinterpret_cast<int*>(base + prep.dy_bytes + prep.w_bytes) : nullptr;
    int rc = prep_dgrad_dy(dy, dydt, base, f.B, f.Tp, prep.Cout, f.Cout, f.y_pitch, f.y_halo, ABI_SLACK_ZERO, st, tickets,
                           tickets ? (int)(DGRAD_TICKET_BYTES / 4) : 0);
    if (rc) return rc;
    const void* wp = w;
    if (prep.copy_w) {
        rc = prep_dgrad_w(w, base + prep.dy_bytes, prep.Cout, prep.k, prep.Cin, f.Cout, f.k, prep.s, st);
        if (rc) return rc;
        wp = base + prep.dy_bytes;
    }
    return conv_dgrad_mfma(f, base, wp, dx, tickets, prep.split_bytes, st, tickets != nullptr);
}
}  // namespace w2l

extern "C" size_t w2l_conv1d_bwd_data_workspace_bytes(int B, int T, int Cin, int Cout, int k, int stride, int dtype)
{
    if (check_conv_shape(B, T, Cin, Cout, k, stride)) return 0;
    const DgradPrep p = dgrad_prep(B, T, Cin, Cout, k, stride, dtype);
    return p.ok ? p.total() : 0;
}

extern "C" int w2l_conv1d_bwd_data(const void* dy, const void* w, void* dx, int B, int T, int Cin, int Cout,
                                   int k, int stride, int dtype, int dy_dtype, void* workspace, size_t ws_bytes,
                                   void* stream)
{
    if (!dy || !w || !dx) return W2L_ERR_NULL;
    int rc = check_conv_shape(B, T, Cin, Cout, k, stride);
    if (rc) return rc;
    if (!valid_dtype(dtype) || !valid_dtype(dy_dtype) || (dtype == W2L_F32 && dy_dtype != W2L_F32))
        return W2L_ERR_DTYPE;
    if (!aligned16(dy) || !aligned16(w) || !aligned16(dx)) return W2L_ERR_ALIGN;
    const size_t need = w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, stride, dtype);
    if (workspace && !ws_ok(workspace, ws_bytes, need)) return W2L_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (workspace && need) {
        // dy staged as bf16 into the haloed layout (channels padded to whole blocks of 64), weights copied padded /
        // with the stride folded where the layer needs it: every bf16 shape the MFMA kernels can be brought to.
        // (A 1x1 layer with bf16 dy and whole channel blocks needs none of it: the kernels read its dense dy as it is.)
        const DgradPrep p = dgrad_prep(B, T, Cin, Cout, k, stride, dtype);
        const bool plain_1x1 = k == 1 && stride == 1 && dy_dtype == W2L_BF16 && !p.copy_w;
        if (!plain_1x1) return conv_dgrad_prepared(p, dy, dy_dtype, w, dx, workspace, st);
    }
    return conv_dgrad(dense_desc(B, T, Cin, Cout, k, stride), dy, w, dx, dtype, dy_dtype, st);
}

extern "C" size_t w2l_conv1d_bwd_weight_workspace_bytes(int B, int T, int Cin, int Cout, int k, int stride,
                                                        int dtype)
{
    if (check_conv_shape(B, T, Cin, Cout, k, stride)) return 0;
    size_t n = conv_wgrad_scratch_bytes(Cin, Cout, k);
    ConvDesc f;
    if (stage_wgrad(Cin, Cout, k, stride, dtype)) n += haloed_bytes(B, T, Cin) + haloed_bytes(B, T, Cout);
    else if (stage_wgrad_folded(B, T, Cin, Cout, k, stride, dtype, f)) n += haloed_bytes(B, f.T, f.Cin) + haloed_bytes(B, f.T, Cout);
    return n;
}

extern "C" int w2l_conv1d_bwd_weight(const void* x, const void* dy, float* dw, float* dbias, int B, int T,
                                     int Cin, int Cout, int k, int stride, int dtype, int dy_dtype,
                                     int accumulate, void* workspace, size_t ws_bytes, void* stream)
{
    if (!x || !dy || !dw) return W2L_ERR_NULL;
    int rc = check_conv_shape(B, T, Cin, Cout, k, stride);
    if (rc) return rc;
    if (!valid_dtype(dtype) || !valid_dtype(dy_dtype) || (dtype == W2L_F32 && dy_dtype != W2L_F32))
        return W2L_ERR_DTYPE;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dw) || (dbias && !aligned16(dbias))) return W2L_ERR_ALIGN;
    if (!ws_ok(workspace, ws_bytes, w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, stride, dtype)))
        return W2L_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    ConvDesc d = dense_desc(B, T, Cin, Cout, k, stride);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    ConvDesc f;
    if (dy_dtype == W2L_BF16 && stage_wgrad_folded(B, T, Cin, Cout, k, stride, dtype, f)) {
        unsigned char* xp = ws + conv_wgrad_scratch_bytes(Cin, Cout, k);
        unsigned char* dyp = xp + haloed_bytes(B, f.T, f.Cin);
        rc = pad_layout2_bf16(x, xp, f.Cin, dy, dyp, Cout, B, f.T, f.T + 2 * ABI_HALO, ABI_HALO, ABI_SLACK_ZERO, st);
        if (rc) return rc;
        f.x_pitch = f.y_pitch = f.T + 2 * ABI_HALO;
        f.x_halo = f.y_halo = ABI_HALO;
        f.slack = ABI_SLACK;
        return conv_wgrad(f, xp, dyp, dw, dbias, dtype, dy_dtype, accumulate, workspace, st);
    }
    if (dy_dtype == W2L_BF16 && stage_wgrad(Cin, Cout, k, stride, dtype)) {
        unsigned char* xp = ws + conv_wgrad_scratch_bytes(Cin, Cout, k);
        unsigned char* dyp = xp + haloed_bytes(B, T, Cin);
        rc = pad_layout2_bf16(x, xp, Cin, dy, dyp, Cout, B, T, T + 2 * ABI_HALO, ABI_HALO, ABI_SLACK_ZERO, st);
        if (rc) return rc;
        d.x_pitch = d.y_pitch = T + 2 * ABI_HALO;
        d.x_halo = d.y_halo = ABI_HALO;
        d.slack = ABI_SLACK;
        x = xp;
        dy = dyp;
    }
    return conv_wgrad(d, x, dy, dw, dbias, dtype, dy_dtype, accumulate, workspace, st);
}

// ---- measurement aid: what the matrix pipe sustains with nothing else going on -----------
namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned probe_u32x4;
// RANDOM: operands with random sign and mantissa bits (what real activations look like to the multipliers);
// otherwise small integers.  The part is power-limited, and the power of the matrix pipe depends on how many
// operand bits toggle: the two settings sustain different clocks.
template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_probe_k(float* out, int iters)
{
    probe_f32x16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    probe_u32x4 a[4], b[4];
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int q = 0; q < 4; ++q)
        for (int e = 0; e < 4; ++e) {
            h = h * 1664525u + 1013904223u;
            unsigned va = h;
            h = h * 1664525u + 1013904223u;
            unsigned vb = h;
            if (RANDOM) {  // two bf16 per word: random sign and mantissa, magnitude in [0.5, 1)
                va = (va & 0x807f807fu) | 0x3f003f00u;
                vb = (vb & 0x807f807fu) | 0x3f003f00u;
            } else {       // 1.0 and 2.0 everywhere
                va = 0x3f803f80u;
                vb = 0x40004000u;
            }
            a[q][e] = va;
            b[q][e] = vb;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(probe_bf16x8, a[i & 3]),
                                                             __builtin_bit_cast(probe_bf16x8, b[(i + it) & 3]), acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace

extern "C" int w2l_probe_mfma(float* out, int blocks, int iters, int random_operands, void* stream)
{
    if (!out) return W2L_ERR_NULL;
    if (blocks <= 0 || blocks > 65535 || iters <= 0) return W2L_ERR_SHAPE;
    if (random_operands) hipLaunchKernelGGL(mfma_probe_k<true>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
    else hipLaunchKernelGGL(mfma_probe_k<false>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
    return launch_status();
}
