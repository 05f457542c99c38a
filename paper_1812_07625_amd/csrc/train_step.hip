// One training step of the conv-GLU network with the CTC criterion, sequenced on one
// stream with no host synchronisation (paper Sec. 2.3: network forward, criterion,
// backward; the optimiser update is a separate stage of the paper's loop, Sec. 2.4).
//
//   forward   for each layer: conv1d(+bias) -> [GLU]      (pre-GLU and post-GLU kept)
//   criterion log-softmax + CTC on the fp32 logits; yields d loss / d logits directly
//   backward  for each layer, last to first: [GLU bwd] -> wgrad(+dbias) -> dgrad
//             (dgrad is skipped for layer 0: the features need no gradient)
#include <vector>
#include "common.h"

namespace w2l {
namespace {

struct Plan {
    int n = 0, C = 0, Tlast = 0, tot_stride = 1;
    std::vector<int> Tin, Tout, outch;
    std::vector<size_t> pre, post;  // workspace offsets of conv output and GLU output per layer
    size_t dlogits = 0, crit_len = 0, gbuf0 = 0, gbuf1 = 0, ctc = 0, conv = 0, total = 0;
    size_t ctc_bytes = 0, conv_bytes = 0;
    int status = W2L_OK;
};

Plan make_plan(const w2l_layer* L, int n, int B, int T, int Lmax, int dtype)
{
    Plan p;
    p.n = n;
    if (!L) { p.status = W2L_ERR_NULL; return p; }
    if (n <= 0 || n > 1024 || B <= 0 || T <= 0 || Lmax <= 0) { p.status = W2L_ERR_SHAPE; return p; }
    if (!valid_dtype(dtype)) { p.status = W2L_ERR_DTYPE; return p; }
    const size_t es = dtype_size(dtype);
    size_t off = 0, gmax = 0;
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
            off += round_up((size_t)B * to * (l.cout / 2) * es, 256);
        } else {
            p.post.push_back(p.pre.back());
        }
        const size_t g1 = (size_t)B * to * l.cout * 4, g2 = (size_t)B * t * l.cin * 4;
        gmax = g1 > gmax ? g1 : gmax;
        gmax = g2 > gmax ? g2 : gmax;
        const size_t cw = w2l_conv1d_bwd_weight_workspace_bytes(B, t, l.cin, l.cout, l.k, l.stride, dtype);
        p.conv_bytes = cw > p.conv_bytes ? cw : p.conv_bytes;
        t = to;
    }
    p.Tlast = t;
    p.C = L[n - 1].cout;
    p.dlogits = off; off += round_up((size_t)B * p.Tlast * p.C * 4, 256);
    p.crit_len = off; off += round_up((size_t)B * 4, 256);
    p.gbuf0 = off; off += round_up(gmax, 256);
    p.gbuf1 = off; off += round_up(gmax, 256);
    p.ctc_bytes = w2l_ctc_workspace_bytes(B, p.Tlast, p.C, Lmax);
    p.ctc = off; off += round_up(p.ctc_bytes, 256);
    p.conv = off; off += round_up(p.conv_bytes, 256);
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
    Plan p = make_plan(layers, n_layers, B, T, Lmax, dtype);
    return p.status == W2L_OK ? p.total : 0;
}

extern "C" int w2l_train_step(const w2l_layer* layers, int n_layers, const void* const* weights,
                              const float* const* biases, float* const* dweights, float* const* dbiases,
                              const void* x, const int* in_len, const int* targets, const int* tgt_len,
                              float* loss, float* logits, int B, int T, int Lmax, int blank, int dtype,
                              float grad_scale, void* workspace, size_t ws_bytes, void* stream)
{
    if (!layers || !weights || !biases || !dweights || !dbiases || !x || !in_len || !targets || !tgt_len || !loss)
        return W2L_ERR_NULL;
    Plan p = make_plan(layers, n_layers, B, T, Lmax, dtype);
    if (p.status) return p.status;
    if (blank < 0 || blank >= p.C) return W2L_ERR_SHAPE;
    for (int i = 0; i < n_layers; ++i)
        if (!weights[i] || !dweights[i]) return W2L_ERR_NULL;
    if (!workspace || ws_bytes < p.total || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return W2L_ERR_WORKSPACE;
    if (!aligned16(x)) return W2L_ERR_ALIGN;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    hipStream_t st = (hipStream_t)stream;
    const int n = n_layers;
    int rc;

    // ---- network forward
    const void* h = x;
    for (int i = 0; i < n; ++i) {
        const w2l_layer& l = layers[i];
        const int ydt = (i == n - 1) ? W2L_F32 : dtype;
        rc = w2l_conv1d_fwd(h, weights[i], biases[i], ws + p.pre[i], B, p.Tin[i], l.cin, l.cout, l.k, l.stride,
                            dtype, ydt, nullptr, 0, stream);
        if (rc) return rc;
        if (l.glu) {
            rc = w2l_glu_fwd(ws + p.pre[i], ws + p.post[i], (long long)B * p.Tout[i], l.cout, dtype, stream);
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
    int* clen = reinterpret_cast<int*>(ws + p.crit_len);
    hipLaunchKernelGGL(crit_len_k, dim3((B + 255) / 256), dim3(256), 0, st, in_len, clen, B, p.tot_stride);
    rc = launch_status();
    if (rc) return rc;
    float* dz = reinterpret_cast<float*>(ws + p.dlogits);
    rc = w2l_ctc_fwd_bwd(z, 1, targets, clen, tgt_len, loss, dz, B, p.Tlast, p.C, Lmax, blank, grad_scale,
                         ws + p.ctc, p.ctc_bytes, stream);
    if (rc) return rc;

    // ---- backward
    void* gb[2] = {ws + p.gbuf0, ws + p.gbuf1};
    const void* dh = dz;  // gradient wrt layer i's (post-GLU) output
    int dh_dt = W2L_F32;
    int cur = 0;          // buffer free to write next
    for (int i = n - 1; i >= 0; --i) {
        const w2l_layer& l = layers[i];
        const void* dy = dh;
        int dy_dt = dh_dt;
        if (l.glu) {
            // dh arrives in the activation dtype for every GLU layer (it was written by a dgrad)
            rc = w2l_glu_bwd(ws + p.pre[i], dh, gb[cur], (long long)B * p.Tout[i], l.cout, dtype, stream);
            if (rc) return rc;
            dy = gb[cur];
            dy_dt = dtype;
            cur ^= 1;
        }
        const void* xin = (i == 0) ? x : (const void*)(ws + p.post[i - 1]);
        rc = w2l_conv1d_bwd_weight(xin, dy, dweights[i], dbiases[i], B, p.Tin[i], l.cin, l.cout, l.k, l.stride,
                                   dtype, dy_dt, 0, ws + p.conv, p.conv_bytes, stream);
        if (rc) return rc;
        if (i > 0) {
            // write into the buffer that does not hold dy
            void* out = (dy == gb[0]) ? gb[1] : gb[0];
            rc = w2l_conv1d_bwd_data(dy, weights[i], out, B, p.Tin[i], l.cin, l.cout, l.k, l.stride, dtype, dy_dt,
                                     nullptr, 0, stream);
            if (rc) return rc;
            dh = out;
            dh_dt = dtype;
            cur = (out == gb[0]) ? 1 : 0;
        }
    }
    return W2L_OK;
}
