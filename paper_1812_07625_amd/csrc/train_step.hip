// One training step of the conv-GLU network with the CTC criterion, sequenced on one
// stream with no host synchronisation (paper Sec. 2.3: network forward, criterion,
// backward; the optimiser update is a separate stage of the paper's loop, Sec. 2.4).
//
//   forward   for each layer: conv1d(+bias) -> [GLU]      (pre-GLU and post-GLU kept)
//   criterion log-softmax + CTC on the fp32 logits; yields d loss / d logits directly
//   backward  for each layer, last to first: [GLU bwd] -> wgrad(+dbias) -> dgrad
//             (dgrad is skipped for layer 0: the features need no gradient)
#include <mutex>
#include <vector>
#include "common.h"

namespace w2l {
namespace {

// Activations that feed a convolution (GLU outputs h_i, and the gradients dy_i that feed
// dgrad/wgrad) are kept with HALO zero frames around every utterance and SLACK zero frames
// after the last one, so the convolution kernels can read every window as plain memory.
// Tensors only read elementwise (pre-GLU outputs y_i, gradients dh_i) stay dense.
constexpr int HALO = LAYOUT_HALO;
constexpr int SLACK = LAYOUT_SLACK;            // allocated after the last utterance
constexpr int SLACK_ZERO = LAYOUT_SLACK_ZERO;  // of which kept zero

// A helper stream (default priority) on which the weight gradients run: wgrad of layer i needs
// only dy_i and h_{i-1}, nothing downstream needs it before the step ends, and neither wgrad
// nor dgrad fills all 256 CUs with its tile grid alone -- side by side they do.  Created once
// per device on first use; no device memory is allocated.
struct SideStream {
    hipStream_t stream = nullptr;
    std::vector<hipEvent_t> ready, done;  // per layer: dy_i written (main) / wgrad_i finished (side)
    bool ok = false;
};
SideStream* side_stream(int n_layers)
{
    static std::mutex mu;
    static SideStream per_device[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    SideStream& s = per_device[dev];
    if (!s.stream) {
        if (hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) != hipSuccess) { s.stream = nullptr; return nullptr; }
        s.ok = true;
    }
    while (s.ok && (int)s.ready.size() < n_layers) {
        hipEvent_t a, b;
        if (hipEventCreateWithFlags(&a, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&b, hipEventDisableTiming) != hipSuccess) { s.ok = false; break; }
        s.ready.push_back(a);
        s.done.push_back(b);
    }
    return s.ok ? &s : nullptr;
}

enum { CRIT_CTC = 0, CRIT_ASG = 1 };

struct Plan {
    int n = 0, C = 0, Tlast = 0, tot_stride = 1;
    std::vector<int> Tin, Tout, outch;
    std::vector<size_t> pre, post;  // workspace offsets of conv output (dense) and GLU output (haloed) per layer
    size_t dlogits = 0, crit_len = 0, gdy[3] = {0, 0, 0}, gdh[2] = {0, 0}, ctc = 0, conv = 0, conv0 = 0, dbias = 0, dgs = 0, total = 0;
    size_t ctc_bytes = 0, conv_bytes = 0, dgs_bytes = 0;
    size_t xfold = 0;      // haloed copy of x with the first layer's stride folded into the channels (0 bytes if unused)
    bool fold0 = false;
    size_t cls = 0;        // operands of the last layer's data gradient prepared for the MFMA kernels (its dy is fp32)
    DgradPrep cls_prep;
    int status = W2L_OK;
};

size_t haloed_bytes(int B, int frames, int ch, size_t es) { return ((size_t)B * (frames + 2 * HALO) + SLACK) * ch * es; }

Plan make_plan(const w2l_layer* L, int n, int B, int T, int Lmax, int dtype, int criterion)
{
    Plan p;
    p.n = n;
    if (!L) { p.status = W2L_ERR_NULL; return p; }
    if (n <= 0 || n > 1024 || B <= 0 || T <= 0 || Lmax <= 0) { p.status = W2L_ERR_SHAPE; return p; }
    if (!valid_dtype(dtype)) { p.status = W2L_ERR_DTYPE; return p; }
    const size_t es = dtype_size(dtype);
    size_t off = 0, dymax = 0, dhmax = 0;
    int t = T;
    for (int i = 0; i < n; ++i) {
        const w2l_layer& l = L[i];
        if (l.k <= 0 || (l.k & 1) == 0 || l.stride <= 0 || l.cin <= 0 || l.cout <= 0) { p.status = W2L_ERR_SHAPE; return p; }
        if (l.glu && (l.cout & 1)) { p.status = W2L_ERR_SHAPE; return p; }
        if (i == n - 1 && l.glu) { p.status = W2L_ERR_SHAPE; return p; }
        if (i > 0 && l.cin != p.outch[i - 1]) { p.status = W2L_ERR_SHAPE; return p; }
        const int to = out_len(t, l.stride);
        p.Tin.push_back(t);
        p.Tout.push_back(to);
        p.outch.push_back(l.glu ? l.cout / 2 : l.cout);
        p.tot_stride *= l.stride;
        const size_t oes = (i == n - 1) ? 4 : es;  // logits are fp32
        p.pre.push_back(off);
        off += round_up((size_t)B * to * l.cout * oes, 256);
        if (l.glu) {
            p.post.push_back(off);
            off += round_up(haloed_bytes(B, to, l.cout / 2, es), 256);
            const size_t g1 = haloed_bytes(B, to, l.cout, es);
            dymax = g1 > dymax ? g1 : dymax;
        } else if (i < n - 1) {
            // a layer without GLU that feeds another layer: its output is copied into the haloed layout too
            p.post.push_back(off);
            off += round_up(haloed_bytes(B, to, l.cout, es), 256);
        } else {
            p.post.push_back(p.pre.back());
        }
        const size_t g2 = (size_t)B * t * l.cin * es;
        dhmax = g2 > dhmax ? g2 : dhmax;
        const size_t cw = w2l_conv1d_bwd_weight_workspace_bytes(B, t, l.cin, l.cout, l.k, l.stride, dtype);
        p.conv_bytes = cw > p.conv_bytes ? cw : p.conv_bytes;
        if (i > 0 && L[i - 1].glu) {
            // scratch of a split-reduction data gradient (tickets and the fp32 sums of both halves)
            ConvDesc sd = dense_desc(B, t, l.cin, l.cout, l.k, l.stride);
            sd.x_pitch = sd.y_pitch = to + 2 * HALO;
            sd.x_halo = sd.y_halo = HALO;
            sd.slack = SLACK;
            const size_t sb = conv_dgrad_scratch_bytes(sd);
            p.dgs_bytes = sb > p.dgs_bytes ? sb : p.dgs_bytes;
        }
        t = to;
    }
    p.Tlast = t;
    p.C = L[n - 1].cout;
    p.dlogits = off; off += round_up((size_t)B * p.Tlast * p.C * 4, 256);
    p.crit_len = off; off += round_up((size_t)B * 4, 256);
    for (int q = 0; q < 3; ++q) { p.gdy[q] = off; off += round_up(dymax, 256); }
    for (int q = 0; q < 2; ++q) { p.gdh[q] = off; off += round_up(dhmax, 256); }
    p.ctc_bytes = criterion == CRIT_ASG ? w2l_asg_workspace_bytes(B, p.Tlast, p.C, Lmax) : w2l_ctc_workspace_bytes(B, p.Tlast, p.C, Lmax);
    if (p.ctc_bytes == 0) { p.status = W2L_ERR_SHAPE; return p; }  // more classes or labels than the criterion takes
    p.ctc = off; off += round_up(p.ctc_bytes, 256);
    p.conv = off; off += round_up(p.conv_bytes, 256);
    // layer 0's weight gradient runs on the caller's stream next to the helper stream's launches: its own scratch
    p.conv0 = off; off += round_up(conv_wgrad_scratch_bytes(L[0].cin, L[0].cout, L[0].k), 256);
    int cmax = 0;
    for (int i = 0; i < n; ++i) cmax = L[i].cout > cmax ? L[i].cout : cmax;
    p.dbias = off; off += round_up((size_t)DBIAS_CHUNKS * cmax * 4, 256);
    p.dgs = off; off += round_up(p.dgs_bytes, 256);
    {
        // a strided first layer with GLU (its dy is haloed): the weight gradient reads x folded and haloed
        ConvDesc d0 = dense_desc(B, T, L[0].cin, L[0].cout, L[0].k, L[0].stride), f0;
        p.fold0 = dtype == W2L_BF16 && L[0].glu && n > 1 && fold_stride(d0, f0) && f0.p <= HALO && f0.Cin % 8 == 0 &&
                  L[0].cout >= 64;
        p.xfold = off;
        if (p.fold0) off += round_up(haloed_bytes(B, f0.T, f0.Cin, es), 256);
    }
    if (n > 1) {
        const w2l_layer& ll = L[n - 1];
        p.cls_prep = dgrad_prep(B, p.Tin[n - 1], ll.cin, ll.cout, ll.k, ll.stride, dtype);
        p.cls = off;
        if (p.cls_prep.ok) off += round_up(p.cls_prep.total(), 256);
    }
    p.total = off;
    return p;
}

__global__ void crit_len_k(const int* in_len, int* out, int B, int tot_stride)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) {
        const int n = in_len[b];
        out[b] = n < 0 ? n : (n + tot_stride - 1) / tot_stride;
    }
}

}  // namespace
}  // namespace w2l

using namespace w2l;

extern "C" size_t w2l_train_step_workspace_bytes(const w2l_layer* layers, int n_layers, int B, int T, int Lmax,
                                                 int dtype)
{
    Plan p = make_plan(layers, n_layers, B, T, Lmax, dtype, CRIT_CTC);
    return p.status == W2L_OK ? p.total : 0;
}

extern "C" size_t w2l_train_step_asg_workspace_bytes(const w2l_layer* layers, int n_layers, int B, int T, int Lmax,
                                                     int dtype)
{
    Plan p = make_plan(layers, n_layers, B, T, Lmax, dtype, CRIT_ASG);
    return p.status == W2L_OK ? p.total : 0;
}

// network forward, criterion (CTC on the log-softmax of the output, or ASG on the output itself), backward
static int train_step_impl(int criterion, const w2l_layer* layers, int n_layers, const void* const* weights,
                           const float* const* biases, float* const* dweights, float* const* dbiases, const void* x,
                           const int* in_len, const int* targets, const int* tgt_len, const float* trans, float* dtrans,
                           float* loss, float* logits, int B, int T, int Lmax, int blank, int dtype, float grad_scale,
                           void* workspace, size_t ws_bytes, void* stream)
{
    if (!layers || !weights || !biases || !dweights || !dbiases || !x || !in_len || !targets || !tgt_len || !loss)
        return W2L_ERR_NULL;
    if (criterion == CRIT_ASG && !trans) return W2L_ERR_NULL;
    Plan p = make_plan(layers, n_layers, B, T, Lmax, dtype, criterion);
    if (p.status) return p.status;
    if (criterion == CRIT_CTC && (blank < 0 || blank >= p.C)) return W2L_ERR_SHAPE;
    for (int i = 0; i < n_layers; ++i)
        if (!weights[i] || !dweights[i]) return W2L_ERR_NULL;
    if (!workspace || ws_bytes < p.total || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return W2L_ERR_WORKSPACE;
    if (!aligned16(x)) return W2L_ERR_ALIGN;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    hipStream_t st = (hipStream_t)stream;
    const int n = n_layers;
    int rc;

    // geometry of layer i; its input is the caller's dense x (i = 0) or the haloed h_{i-1}
    auto desc = [&](int i) {
        const w2l_layer& l = layers[i];
        ConvDesc d = dense_desc(B, p.Tin[i], l.cin, l.cout, l.k, l.stride);
        if (i > 0) { d.x_pitch = p.Tin[i] + 2 * HALO; d.x_halo = HALO; d.slack = SLACK; }
        return d;
    };

    // ---- network forward: y_i = conv(h_{i-1}) + bias (dense), h_i = GLU(y_i) (haloed)
    const void* h = x;
    for (int i = 0; i < n; ++i) {
        const w2l_layer& l = layers[i];
        const int ydt = (i == n - 1) ? W2L_F32 : dtype;
        const ConvDesc fd = desc(i);
        if (l.glu && dtype == W2L_BF16 && ydt == W2L_BF16 && conv_fwd_glu_ok(fd)) {
            rc = conv_fwd_glu(fd, h, weights[i], biases[i], ws + p.pre[i], ws + p.post[i], st);  // GLU in the epilogue
            if (rc) return rc;
            h = ws + p.post[i];
            continue;
        }
        rc = conv_fwd(fd, h, weights[i], biases[i], ws + p.pre[i], dtype, ydt, st);
        if (rc) return rc;
        if (l.glu) {
            rc = glu_fwd_layout(ws + p.pre[i], ws + p.post[i], B, p.Tout[i], l.cout, dtype, p.Tout[i] + 2 * HALO, HALO,
                                SLACK_ZERO, st);
            if (rc) return rc;
        } else if (i < n - 1) {
            rc = pad_layout(ws + p.pre[i], ws + p.post[i], B, p.Tout[i], l.cout, dtype, p.Tout[i] + 2 * HALO, HALO,
                            SLACK_ZERO, st);
            if (rc) return rc;
        }
        h = ws + p.post[i];
    }
    const float* z = reinterpret_cast<const float*>(ws + p.pre[n - 1]);
    if (logits) {
        hipError_t e = hipMemcpyAsync(logits, z, (size_t)B * p.Tlast * p.C * 4, hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    }

    // ---- criterion: frames seen = ceil(in_len / total stride)
    float* dz = reinterpret_cast<float*>(ws + p.dlogits);
    if (criterion == CRIT_ASG) {
        int* clen = reinterpret_cast<int*>(ws + p.crit_len);
        hipLaunchKernelGGL(crit_len_k, dim3((B + 255) / 256), dim3(256), 0, st, in_len, clen, B, p.tot_stride);
        rc = launch_status();
        if (rc) return rc;
        rc = w2l_asg_fwd_bwd(z, trans, targets, clen, tgt_len, loss, dz, dtrans, B, p.Tlast, p.C, Lmax, grad_scale,
                             ws + p.ctc, p.ctc_bytes, stream);
    } else {
        rc = ctc_fwd_bwd_strided(z, 1, targets, in_len, tgt_len, loss, dz, B, p.Tlast, p.C, Lmax, blank, grad_scale,
                                 ws + p.ctc, p.ctc_bytes, stream, p.tot_stride);
    }
    if (rc) return rc;

    // ---- backward.  dh = gradient wrt layer i's output (dense); dy = gradient wrt its conv
    // output: the haloed result of the GLU backward, or dh itself for a layer without GLU.
    // Main stream: the dgrad chain.  Where the shapes allow, the data gradient of layer i applies
    // the GLU backward of layer i-1 in its epilogue and writes dy_{i-1} directly; otherwise dh
    // goes to memory and a GLU-backward kernel follows.  Side stream: wgrad (+dbias) of every
    // layer, each started as soon as its dy exists.  dy buffers rotate over three slots, so the
    // writer of dy_i only has to wait for the weight gradient of layer i+3.
    SideStream* side = side_stream(n);
    auto hip_ok = [&](hipError_t e) { if (e != hipSuccess) { note_hip_error(e); return false; } return true; };
    auto wait_wgrad = [&](int layer) {  // main stream waits until that layer's weight gradient has read its dy
        if (!side || layer >= n) return true;
        return hip_ok(hipStreamWaitEvent(st, side->done[layer], 0));
    };
    // dh tensors that go to memory alternate between two buffers: a layer without GLU takes dh itself as its dy,
    // so its data gradient must not write the buffer it reads, nor one the helper stream's weight gradient
    // of the layer above still reads (gdh_reader: that layer, or -1)
    void* const gdhb[2] = {ws + p.gdh[0], ws + p.gdh[1]};
    int gdh_reader[2] = {-1, -1};
    int cur = -1;  // the buffer that holds dh; -1: dh is the criterion's gradient
    const void* dh = dz;
    int dh_dt = W2L_F32;
    bool dy_ready = false;  // dy of the current layer was already written by the layer above
    for (int i = n - 1; i >= 0; --i) {
        const w2l_layer& l = layers[i];
        ConvDesc d = desc(i);
        const void* dy = dh;
        int dy_dt = dh_dt;
        if (l.glu) {
            void* gdy = ws + p.gdy[i % 3];
            if (!dy_ready) {
                if (!wait_wgrad(i + 3)) return W2L_ERR_LAUNCH;
                rc = glu_bwd_layout(ws + p.pre[i], dh, gdy, B, p.Tout[i], l.cout, dtype, p.Tout[i] + 2 * HALO, HALO,
                                    SLACK_ZERO, st);
                if (rc) return rc;
            }
            dy = gdy;
            dy_dt = dtype;
            d.y_pitch = p.Tout[i] + 2 * HALO;
            d.y_halo = HALO;
            d.slack = SLACK;
        } else {
            d.slack = 0;  // dy is dense here: nothing may be read past its end
            if (side && i > 0 && cur >= 0) gdh_reader[cur] = i;
        }
        dy_ready = false;
        // layer 0 has no data gradient: its weight gradient takes the main stream, next to the
        // helper stream's last launch, instead of queueing behind it
        const bool on_side = side && i > 0;
        hipStream_t wst = on_side ? side->stream : st;
        if (on_side) {
            if (!hip_ok(hipEventRecord(side->ready[i], st)) || !hip_ok(hipStreamWaitEvent(wst, side->ready[i], 0)))
                return W2L_ERR_LAUNCH;
        }
        const void* xin = (i == 0) ? x : (const void*)(ws + p.post[i - 1]);
        if (i == 0 && p.fold0) {
            // the strided first layer as a stride-1 layer over folded frames: x copied (2 MB) into the haloed time
            // layout of dy_0, then the same dense weight-gradient kernel as every other layer, bias gradient included
            ConvDesc f;
            fold_stride(dense_desc(B, p.Tin[0], l.cin, l.cout, l.k, l.stride), f);
            f.x_pitch = f.y_pitch = p.Tout[0] + 2 * HALO;
            f.x_halo = f.y_halo = HALO;
            f.slack = SLACK;
            rc = pad_layout_bf16(x, ws + p.xfold, B, f.T, f.Cin, f.x_pitch, HALO, SLACK_ZERO, st);
            if (rc) return rc;
            d = f;
            xin = ws + p.xfold;
        }
        // weight gradient on the side stream.  Where the MFMA kernel takes it, the bias gradient is one more
        // column of tiles of the same launch; otherwise it is a (small, bandwidth-bound) column sum that stays
        // on the main stream, which has the shorter chain
        const bool fused_dbias = dbiases[i] && conv_wgrad_fuses_dbias(d, dtype, dy_dt);
        rc = conv_wgrad(d, xin, dy, dweights[i], (fused_dbias || !side) ? dbiases[i] : nullptr, dtype, dy_dt, 0,
                        ws + (i == 0 ? p.conv0 : p.conv), wst);
        if (rc) return rc;
        if (on_side && !hip_ok(hipEventRecord(side->done[i], wst))) return W2L_ERR_LAUNCH;
        if (side && dbiases[i] && !fused_dbias) {
            // halo frames hold zeros, so summing every frame of the allocation is the same sum
            rc = dbias_reduce(dy, dbiases[i], (long long)d.B * d.y_pitch, d.Cout, dy_dt, 0,
                              reinterpret_cast<float*>(ws + p.dbias), st);
            if (rc) return rc;
        }
        if (i > 0) {
            if (layers[i - 1].glu && dtype == W2L_BF16 && dy_dt == W2L_BF16 && conv_dgrad_glu_ok(d)) {
                if (!wait_wgrad(i + 2)) return W2L_ERR_LAUNCH;  // last reader of the slot dy_{i-1} goes into
                rc = conv_dgrad_glu(d, dy, weights[i], ws + p.pre[i - 1], ws + p.gdy[(i - 1) % 3], ws + p.dgs, p.dgs_bytes, st);
                if (rc) return rc;
                dy_ready = true;
                continue;
            }
            ConvDesc dd = d;   // dx = dh_{i-1} is written dense
            dd.x_pitch = p.Tin[i];
            dd.x_halo = 0;
            const int q = (cur == 0) ? 1 : 0;
            if (gdh_reader[q] >= 0) {
                if (!wait_wgrad(gdh_reader[q])) return W2L_ERR_LAUNCH;
                gdh_reader[q] = -1;
            }
            if (i == n - 1 && dy_dt == W2L_F32 && p.cls_prep.ok)  // the criterion's fp32 gradient: cast, pad, MFMA
                rc = conv_dgrad_prepared(p.cls_prep, dy, dy_dt, weights[i], gdhb[q], ws + p.cls, st);
            else
                rc = conv_dgrad(dd, dy, weights[i], gdhb[q], dtype, dy_dt, st);
            if (rc) return rc;
            dh = gdhb[q];
            cur = q;
            dh_dt = dtype;
        }
    }
    // join: the side stream is in order, so its last event covers every weight gradient
    if (side && n > 1 && !hip_ok(hipStreamWaitEvent(st, side->done[1], 0))) return W2L_ERR_LAUNCH;
    return W2L_OK;
}

extern "C" int w2l_train_step(const w2l_layer* layers, int n_layers, const void* const* weights,
                              const float* const* biases, float* const* dweights, float* const* dbiases,
                              const void* x, const int* in_len, const int* targets, const int* tgt_len,
                              float* loss, float* logits, int B, int T, int Lmax, int blank, int dtype,
                              float grad_scale, void* workspace, size_t ws_bytes, void* stream)
{
    return train_step_impl(CRIT_CTC, layers, n_layers, weights, biases, dweights, dbiases, x, in_len, targets, tgt_len,
                           nullptr, nullptr, loss, logits, B, T, Lmax, blank, dtype, grad_scale, workspace, ws_bytes, stream);
}

extern "C" int w2l_train_step_asg(const w2l_layer* layers, int n_layers, const void* const* weights,
                                  const float* const* biases, float* const* dweights, float* const* dbiases,
                                  const void* x, const int* in_len, const int* targets, const int* tgt_len,
                                  const float* trans, float* dtrans, float* loss, float* logits, int B, int T, int Lmax,
                                  int dtype, float grad_scale, void* workspace, size_t ws_bytes, void* stream)
{
    return train_step_impl(CRIT_ASG, layers, n_layers, weights, biases, dweights, dbiases, x, in_len, targets, tgt_len,
                           trans, dtrans, loss, logits, B, T, Lmax, 0, dtype, grad_scale, workspace, ws_bytes, stream);
}
