/*
 * w2l.h -- C ABI of libw2l: the forward/backward training step of the paper's
 * all-convolutional grapheme acoustic model with the CTC criterion, as HIP kernels
 * for gfx950 (MI355X), one GPU.
 *
 * The paper (wav2letter++) splits every model into a *network* -- a function of
 * the input only -- and a *criterion* -- a function of the network output and the
 * target transcription (Sec. 2.3).  Here the network is a stack of 1-D temporal
 * convolutions (Sec. 2.3, Sec. 4.1) with bias and gated linear units followed by a
 * per-frame log-softmax, and the criterion is CTC (Sec. 2.3).  The paper names
 * these operations without printing formulas; the exact arithmetic and layout
 * conventions are stated on each entry point below.
 *
 * Conventions common to every call
 *  - All tensor pointers are DEVICE pointers owned by the caller, dense,
 *    row-major ("channels last": x[b][t][c]) and 16-byte aligned.  The library
 *    never allocates or frees device memory; scratch space comes from the
 *    caller's `workspace` (device pointer, 256-byte aligned) whose minimum size
 *    the matching *_workspace_bytes() query returns.  Inputs are never modified.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    enqueue work and return; they never synchronise with the host.  Outputs,
 *    including losses, stay on the device.
 *  - dtype: W2L_F32 or W2L_BF16 (bf16 = upper 16 bits of an IEEE float,
 *    round-to-nearest-even on store).  Accumulation is always fp32; bias, weight
 *    gradients, bias gradients, log-probabilities, losses and CTC gradients are
 *    always fp32.
 *  - Every function returns W2L_OK (0) or a negative w2l_status.  Arguments are
 *    validated on the host before anything is launched; on error nothing is
 *    launched.  The library never throws, aborts or prints.
 *  - Time: T input frames, stride s >= 1, odd kernel width k, symmetric zero
 *    padding p = (k-1)/2, output frames T' = ceil(T/s).
 */
#ifndef W2L_H
#define W2L_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    W2L_OK = 0,
    W2L_ERR_NULL = -1,      /* a required pointer is NULL */
    W2L_ERR_SHAPE = -2,     /* non-positive size, even k, odd Cout with GLU, size over a limit */
    W2L_ERR_DTYPE = -3,     /* unknown or unsupported dtype combination */
    W2L_ERR_ALIGN = -4,     /* a pointer is not 16-byte aligned */
    W2L_ERR_WORKSPACE = -5, /* workspace NULL or smaller than *_workspace_bytes() */
    W2L_ERR_TARGET = -6,    /* (host validation helper) bad label or length */
    W2L_ERR_LAUNCH = -7     /* HIP reported an error; see w2l_last_hip_error() */
} w2l_status;

typedef enum { W2L_F32 = 0, W2L_BF16 = 1 } w2l_dtype;

/* One network layer: conv1d(k, stride, cin -> cout) + bias, then GLU if glu != 0
 * (which halves the channel count seen by the next layer). */
typedef struct {
    int k, stride, cin, cout, glu;
} w2l_layer;

int w2l_version(void);
const char *w2l_status_str(int status);
/* hipError_t value of the most recent failed HIP call made by this library (0 if none). */
int w2l_last_hip_error(void);

/* ---- temporal convolution (Sec. 2.3 "1D convolutions"; Sec. 4.1) ------------------
 * Cross-correlation:
 *   y[b,t',co] = bias[co] + sum_{j<k} sum_{ci<Cin} w[co,j,ci] * x[b, s*t' + j - p, ci]
 * with x = 0 outside 0 <= t < T.   x: [B,T,Cin] (dtype);  w: [Cout,k,Cin] (dtype);
 * bias: [Cout] fp32 or NULL;  y: [B,T',Cout] (y_dtype; W2L_F32 is allowed with bf16
 * operands, e.g. for logits).
 * Workspace is optional for fwd and bwd_data: with NULL the kernels predicate every load
 * against the utterance edges; given the queried number of bytes they first copy the
 * window-read operand into a layout with a zero halo around every utterance (one extra
 * bandwidth-bound pass) and then run the faster unpredicated kernel.  A non-NULL workspace
 * smaller than the query is W2L_ERR_WORKSPACE. */
size_t w2l_conv1d_fwd_workspace_bytes(int B, int T, int Cin, int Cout, int k, int stride, int dtype);
int w2l_conv1d_fwd(const void *x, const void *w, const float *bias, void *y,
                   int B, int T, int Cin, int Cout, int k, int stride,
                   int dtype, int y_dtype, void *workspace, size_t ws_bytes, void *stream);

/* Gradient with respect to the input (transpose of x -> y):
 *   dx[b,t,ci] = sum_j sum_co w[co,j,ci] * dy[b,(t+p-j)/s,co]
 * over taps j with (t+p-j) divisible by s and 0 <= (t+p-j)/s < T'.
 * dy: [B,T',Cout] (dy_dtype);  w: [Cout,k,Cin] (dtype);  dx: [B,T,Cin] (dtype).
 * Given the queried workspace, bf16 problems run on the matrix cores whatever Cout is and also for
 * a stride s > 1 with p % s == 0 and T % s == 0: dy is staged as bf16 (an fp32 dy is rounded to
 * bf16 there) with its channels padded to a multiple of 64, the weights are copied padded and with
 * the stride folded into the channels.  Without workspace, fp32 dy, odd channel counts and strided
 * layers take a shape-agnostic fp32 kernel. */
size_t w2l_conv1d_bwd_data_workspace_bytes(int B, int T, int Cin, int Cout, int k, int stride, int dtype);
int w2l_conv1d_bwd_data(const void *dy, const void *w, void *dx,
                        int B, int T, int Cin, int Cout, int k, int stride,
                        int dtype, int dy_dtype, void *workspace, size_t ws_bytes, void *stream);

/* Gradient with respect to weights and bias (transpose of w -> y):
 *   dw[co,j,ci] = sum_b sum_t' dy[b,t',co] * x[b, s*t' + j - p, ci]
 *   dbias[co]   = sum_b sum_t' dy[b,t',co]
 * x: [B,T,Cin] (dtype);  dy: [B,T',Cout] (dy_dtype);  dw: [Cout,k,Cin] fp32;
 * dbias: [Cout] fp32 or NULL.  accumulate = 0 overwrites dw/dbias, 1 adds to them.
 * Reductions run in a fixed order: results are bit-reproducible run to run.
 * The workspace is required here (reduction scratch, plus the haloed operand copies). */
size_t w2l_conv1d_bwd_weight_workspace_bytes(int B, int T, int Cin, int Cout, int k, int stride, int dtype);
int w2l_conv1d_bwd_weight(const void *x, const void *dy, float *dw, float *dbias,
                          int B, int T, int Cin, int Cout, int k, int stride,
                          int dtype, int dy_dtype, int accumulate,
                          void *workspace, size_t ws_bytes, void *stream);

/* ---- gated linear unit (the gated convnet of Sec. 4.1) -----------------------------
 * y: [rows,Cout], Cout even.  Value half a = y[:, :Cout/2], gate half g = y[:, Cout/2:].
 *   fwd:  h = a * sigmoid(g)                          h: [rows,Cout/2]
 *   bwd:  dy[:, :Cout/2] = dh * sigmoid(g)
 *         dy[:, Cout/2:] = dh * a * sigmoid(g) * (1 - sigmoid(g))
 * All tensors share `dtype`; the arithmetic is fp32. */
int w2l_glu_fwd(const void *y, void *h, long long rows, int Cout, int dtype, void *stream);
int w2l_glu_bwd(const void *y, const void *dh, void *dy, long long rows, int Cout, int dtype,
                void *stream);

/* ---- per-frame log-softmax (normalised scores for the criterion, Sec. 2.3) ---------
 *   fwd:  lp[r,c] = z[r,c] - max_c z[r,:] - log sum_c exp(z[r,c] - max_c z[r,:])
 *   bwd:  dz[r,c] = dlp[r,c] - exp(lp[r,c]) * sum_c dlp[r,:]
 * z: [rows,C] (z_dtype);  lp, dlp, dz: [rows,C] fp32.  1 <= C <= 4096. */
int w2l_logsoftmax_fwd(const void *z, float *lp, long long rows, int C, int z_dtype, void *stream);
int w2l_logsoftmax_bwd(const float *lp, const float *dlp, float *dz, long long rows, int C,
                       void *stream);

/* ---- SGD with momentum (Sec. 4.1: the optimiser of every run in the paper) ---------
 * The paper names the optimiser and does not write the update out; this is the classical
 * heavy-ball form with optional L2 weight decay, elementwise over n values:
 *   v[i] = momentum * v[i] + (grad[i] + weight_decay * w[i])
 *   w[i] = w[i] - lr * v[i]
 *   w_lowp[i] = bf16(w[i])              (only if w_lowp != NULL)
 * w: fp32 master weights, v: fp32 velocity (both updated in place), grad: fp32 (the dw / dbias
 * buffers of w2l_train_step), w_lowp: optional bf16 copy of the updated weights (the tensor the
 * next w2l_train_step reads), round-to-nearest-even.  All device pointers, n >= 0, 16-byte
 * aligned.  Arithmetic is fp32.  Returns W2L_ERR_NULL / _SHAPE / _ALIGN like the other calls. */
int w2l_sgd_momentum_step(float *w, float *v, const float *grad, void *w_lowp, long long n, float lr,
                          float momentum, float weight_decay, void *stream);

/* ---- CTC criterion (Sec. 2.3, after Graves et al. 2006) ---------------------------
 * For utterance b with T_b = in_len[b] valid frames and target l (L_b = tgt_len[b]
 * labels), over the extended sequence l' = (blank, l_1, blank, ..., l_L, blank):
 *   loss[b] = -log sum over all frame labellings that collapse to l of
 *             prod_{t<T_b} exp(lp[b,t,pi_t])            (natural log)
 * computed with the alpha/beta recursions (every state kept as fp32 value x 2^int32, a range
 * no smaller than log-space fp32), and
 *   G[b,t,c] = posterior probability that frame t carries class c given l.
 * in:  input [B,Tp,C] fp32 -- log-probabilities (is_logits = 0) or unnormalised
 *      logits (is_logits = 1: a log-softmax is applied inside);
 *      targets [B,Lmax] int32 (row b uses its first tgt_len[b] entries),
 *      in_len [B] int32 (0..Tp), tgt_len [B] int32 (0..Lmax); blank in [0,C).
 * out: loss [B] fp32;  grad [B,Tp,C] fp32 = grad_scale * d(sum_b loss_b)/d input, i.e.
 *      -grad_scale*G (is_logits = 0) or grad_scale*(softmax - G) (is_logits = 1);
 *      rows t >= in_len[b] are 0.
 * A log-probability of -inf (or below -65536 ln 2) is probability zero.
 * An utterance with no valid alignment gets loss +inf and zero gradient.  A label
 * equal to blank or outside [0,C), or a length outside its range, cannot be
 * reported by an asynchronous call: that utterance gets loss NaN and zero
 * gradient (w2l_ctc_check_targets_host() validates host copies beforehand).
 * Limits: C <= 4096, Lmax <= 3000, Tp <= 8192 (else W2L_ERR_SHAPE). */
size_t w2l_ctc_workspace_bytes(int B, int Tp, int C, int Lmax);
int w2l_ctc_fwd_bwd(const float *input, int is_logits, const int *targets, const int *in_len,
                    const int *tgt_len, float *loss, float *grad,
                    int B, int Tp, int C, int Lmax, int blank, float grad_scale,
                    void *workspace, size_t ws_bytes, void *stream);
/* The same computation for callers that cannot allocate device memory (code under HIP graph
 * capture, serving loops, harnesses that forbid hipMalloc): identical arguments and results, but
 * the scratch space is a static device array inside the library instead of a caller workspace,
 * and the call makes no hipMalloc/hipFree or any other allocating call.
 * Limit: w2l_ctc_workspace_bytes(B, Tp, C, Lmax) <= W2L_CTC_NOALLOC_SCRATCH_BYTES (32 MiB: e.g.
 * B = 8, Tp = 750, Lmax = 150, the criterion of the 100M-parameter network's batch); a larger
 * problem is refused with W2L_ERR_WORKSPACE and nothing is launched.  Every device the library
 * runs on holds one such array until the process ends.  All calls on one device share that
 * device's array: two calls in flight on the same device at the same time (two streams, two host
 * threads) race -- order them on one stream.  The array keeps the previous call's contents;
 * every launch writes what it later reads, so nothing needs clearing.  The first call on a device
 * looks the array's address up (hipGetSymbolAddress) and should be made outside a graph capture.
 * Errors: as w2l_ctc_fwd_bwd; W2L_ERR_LAUNCH if the address lookup fails. */
#define W2L_CTC_NOALLOC_SCRATCH_BYTES (32u << 20)
int w2l_ctc_fwd_bwd_noalloc(const float *input, int is_logits, const int *targets, const int *in_len,
                            const int *tgt_len, float *loss, float *grad,
                            int B, int Tp, int C, int Lmax, int blank, float grad_scale, void *stream);
/* Host-only query: which variant of the alpha/beta kernel w2l_ctc_fwd_bwd launches for C classes
 * and targets of up to Lmax labels -- (blank, label) pairs per lane (1, 2 or 4), score-table values
 * a thread stages per block of frames (2, 4, 8; 0 = scores gathered per lane, large alphabets),
 * frames per block (16 or 12) and threads per workgroup.  For tests and tuning; launches nothing.
 * W2L_ERR_SHAPE for sizes w2l_ctc_fwd_bwd refuses. */
int w2l_ctc_launch_config(int C, int Lmax, int *pairs_per_lane, int *table_values_per_thread,
                          int *frames_per_block, int *threads);
/* HOST pointers.  Returns W2L_ERR_TARGET for a label == blank or outside [0,C),
 * in_len outside [0,Tp] or tgt_len outside [0,Lmax]. */
int w2l_ctc_check_targets_host(const int *targets, const int *in_len, const int *tgt_len,
                               int B, int Tp, int C, int Lmax, int blank);

/* ---- ASG criterion (Sec. 2.3: the original wav2letter AutoSegCriterion, the criterion with
 * learned parameters; the paper cites Collobert et al. 2016 for it and prints no formula --
 * the definition below is this library's reading of that criterion) --------------------
 * No blank and no per-frame normalisation.  For utterance b with T_b = in_len[b] frames,
 * target y_0..y_{L-1} (L = tgt_len[b]), emissions f = emissions[b] and transitions g:
 *   score(pi) = sum_{t<T_b} f[t][pi_t] + sum_{1<=t<T_b} g[pi_t][pi_{t-1}]
 *   FCC  = log sum over all C^T_b frame labellings pi of exp(score(pi))
 *   FAL  = log sum over the alignments pi_t = y_{s_t}, s_0 = 0, s_{T_b-1} = L-1,
 *          s_t - s_{t-1} in {0,1}, of exp(score(pi))
 *   loss[b] = FCC - FAL            (natural log; >= 0)
 * in:  emissions [B,Tp,C] fp32 (unnormalised scores); trans [C,C] fp32, trans[i*C+j] = g[i][j]
 *      = score of class j at one frame being followed by class i at the next;
 *      targets [B,Lmax] int32 (labels in [0,C); equal neighbours are allowed),
 *      in_len [B] int32 (0..Tp), tgt_len [B] int32 (0..Lmax).
 * out: loss [B] fp32;
 *      grad_emissions [B,Tp,C] fp32 = grad_scale * d(sum_b loss_b)/d emissions
 *        = grad_scale * (P_fcc(pi_t = c) - P_fal(pi_t = c)); rows t >= in_len[b] are 0;
 *      grad_trans [C,C] fp32 (nullable: not wanted) = grad_scale * d(sum_b loss_b)/d trans
 *        = grad_scale * sum_b sum_t (P_fcc(pi_t = i, pi_{t-1} = j) - the same under FAL),
 *        summed over the batch in a fixed order (overwritten, not accumulated).
 * An utterance with no alignment (L > T_b, or L = 0 with T_b > 0) gets loss +inf and
 * contributes zero gradients; T_b = 0 and L = 0 gives loss 0.  A label outside [0,C) or a
 * length outside its range cannot be reported by an asynchronous call: that utterance gets
 * loss NaN and zero gradients (w2l_asg_check_targets_host() validates host copies).
 * All device pointers; emissions, targets, grad_emissions 16-byte aligned; workspace of
 * w2l_asg_workspace_bytes() bytes, 256-byte aligned, owned by the caller.
 * Limits: C <= 64, Lmax <= 3000.  Errors: W2L_ERR_NULL / _SHAPE / _ALIGN / _WORKSPACE / _LAUNCH. */
size_t w2l_asg_workspace_bytes(int B, int Tp, int C, int Lmax);
int w2l_asg_fwd_bwd(const float *emissions, const float *trans, const int *targets,
                    const int *in_len, const int *tgt_len, float *loss,
                    float *grad_emissions, float *grad_trans,
                    int B, int Tp, int C, int Lmax, float grad_scale,
                    void *workspace, size_t ws_bytes, void *stream);
/* Host-only query: which variant of the lattice kernel w2l_asg_fwd_bwd launches -- target positions
 * per lane (1, 2 or 4), lanes per class row of the fully connected recursion (32 or 64), the
 * workgroup-size bound it is compiled for (256 or 1024), frames per block (16 or 12), emission-row
 * values a thread stages per block (2 or 8) and threads per workgroup.  For tests and tuning;
 * launches nothing.  W2L_ERR_SHAPE for sizes w2l_asg_fwd_bwd refuses. */
int w2l_asg_launch_config(int C, int Lmax, int *positions_per_lane, int *class_lanes, int *max_threads,
                          int *frames_per_block, int *row_values_per_thread, int *threads);
/* HOST pointers.  Returns W2L_ERR_TARGET for a label outside [0,C), in_len outside [0,Tp]
 * or tgt_len outside [0,Lmax]. */
int w2l_asg_check_targets_host(const int *targets, const int *in_len, const int *tgt_len,
                               int B, int Tp, int C, int Lmax);

/* ---- log-mel filterbank features (Sec. 2.2: log-mels are among the feature types computed on
 * the fly before every network evaluation; Sec. 4.1: 40 per frame feed the networks.  The paper
 * fixes no constant or formula -- this is the library's reading) -----------------------------
 * For utterance b with n = wav_len[b] samples (clamped to [0, Nmax]):
 *   frames   t = 0 .. T_b-1, T_b = 1 + floor((n - win) / hop) (0 if n < win): only frames wholly
 *            inside the signal; frame t covers samples t*hop .. t*hop + win - 1
 *   window   0.54 - 0.46 cos(2 pi i / (win - 1))          (Hamming)
 *   spectrum P[k] = | sum_i x[i] window[i] exp(-2 pi sqrt(-1) i k / nfft) |^2, k = 0 .. nfft/2
 *   mel      n_mels + 2 points equally spaced in m = 2595 log10(1 + f/700) between fmin and fmax;
 *            band j rises linearly in Hz from point j to point j+1 (weight 1) and falls to point
 *            j+2, evaluated at the bin frequencies k * sample_rate / nfft
 *   feature  log( max( sum_k weight_j[k] P[k], floor ) )   (natural log)
 * No pre-emphasis, dither or normalisation.
 * in:  wav [B,Nmax] fp32, wav_len [B] int32.
 * out: feat [B,Tmax,n_mels] (dtype: W2L_F32 or W2L_BF16), rows t >= min(T_b, Tmax) are 0 -- the
 *      layout and padding w2l_train_step expects of x; feat_len [B] int32 = min(T_b, Tmax), the
 *      in_len of that call.
 * All device pointers, no workspace; arithmetic fp32 (mel points in double).
 * Limits: nfft a power of two in [128, 1024], 2 <= win <= nfft, hop >= 1, n_mels <= 255,
 * 0 <= fmin < fmax <= sample_rate/2, floor > 0.  Errors: W2L_ERR_NULL / _SHAPE / _DTYPE / _LAUNCH.
 * w2l_logmel_num_frames: the frame count above, on the host. */
int w2l_logmel_num_frames(int n_samples, int win, int hop);
int w2l_logmel_fwd(const float *wav, const int *wav_len, void *feat, int *feat_len,
                   int B, int Nmax, int Tmax, int n_mels, int sample_rate, int win, int hop,
                   int nfft, float fmin, float fmax, float floor, int dtype, void *stream);

/* ---- one training step: network forward, criterion, backward (Sec. 2.3, Sec. 4.1) --
 * layers[0..n_layers): layer i maps [B,T_i,cin_i] to [B,ceil(T_i/stride_i),cout_i or
 * cout_i/2]; cin_0 is the feature dimension, cin_{i+1} must equal layer i's output
 * channels and the last layer's output channels are the C classes (last layer: glu = 0).
 * x: [B,T,cin_0] (dtype), frames t >= in_len[b] must be zero (the network runs on the
 * padded batch; no re-masking between layers).  The criterion sees
 * ceil(in_len[b] / prod_i stride_i) frames of utterance b.
 * weights[i]: [cout,k,cin] (dtype);  biases[i]: [cout] fp32 (NULL entry = no bias);
 * dweights[i]: [cout,k,cin] fp32, dbiases[i]: [cout] fp32 (NULL entry = not wanted);
 * both are overwritten with the gradient of grad_scale * sum_b loss[b].
 * loss: [B] fp32.  logits (nullable): [B,T_last,C] fp32 copy of the network output.
 * The four pointer tables are HOST arrays of DEVICE pointers; x, in_len, targets,
 * tgt_len, loss, logits are device pointers.  With W2L_BF16, activations and
 * gradients between layers are stored as bf16, the last layer's output (logits), the
 * log-softmax and CTC are fp32.
 * Concurrency: the step runs the weight gradients on one helper stream (default priority,
 * created on first use, one per device, never destroyed) tied to `stream` by events, and is
 * complete in `stream` order when the call's work on `stream` is.  Host threads may call
 * concurrently for different devices; two steps in flight on the SAME device at the same time
 * (two streams or two host threads) share that helper stream and its events and are not
 * supported -- order them on one stream.  Like every call here, steps that share a workspace
 * must not overlap. */
size_t w2l_train_step_workspace_bytes(const w2l_layer *layers, int n_layers, int B, int T,
                                      int Lmax, int dtype);
int w2l_train_step(const w2l_layer *layers, int n_layers,
                   const void *const *weights, const float *const *biases,
                   float *const *dweights, float *const *dbiases,
                   const void *x, const int *in_len, const int *targets, const int *tgt_len,
                   float *loss, float *logits,
                   int B, int T, int Lmax, int blank, int dtype, float grad_scale,
                   void *workspace, size_t ws_bytes, void *stream);

/* The same step with the ASG criterion (Sec. 2.3) in place of log-softmax + CTC: the network
 * output [B,T_last,C] is handed to w2l_asg_fwd_bwd as emissions (C <= 64, no blank).
 * trans: [C,C] fp32 transition scores (device); dtrans: [C,C] fp32 (device, nullable = not
 * wanted), overwritten with the gradient of grad_scale * sum_b loss[b].  Everything else as in
 * w2l_train_step; workspace from w2l_train_step_asg_workspace_bytes (0 if the shape is not
 * supported). */
size_t w2l_train_step_asg_workspace_bytes(const w2l_layer *layers, int n_layers, int B, int T,
                                          int Lmax, int dtype);
int w2l_train_step_asg(const w2l_layer *layers, int n_layers,
                       const void *const *weights, const float *const *biases,
                       float *const *dweights, float *const *dbiases,
                       const void *x, const int *in_len, const int *targets, const int *tgt_len,
                       const float *trans, float *dtrans, float *loss, float *logits,
                       int B, int T, int Lmax, int dtype, float grad_scale,
                       void *workspace, size_t ws_bytes, void *stream);

/* ---- measurement aid (not part of the training path) -----------------------------------
 * Launches `blocks` workgroups of 4 wavefronts, each wavefront issuing 8*iters independent
 * v_mfma_f32_32x32x16_bf16 (32768 FLOP each) and nothing else; out: [blocks*256] fp32 sink.
 * random_operands = 0: every operand element is 1.0 or 2.0; != 0: random sign and mantissa bits,
 * as real activations and weights have.  Timed by the caller, it gives the bf16 MFMA rate the
 * part sustains at its clocks under load -- the practical ceiling next to the published
 * 2.5 PFLOP/s.  The part is power-limited and the matrix pipe's power depends on how many operand
 * bits toggle, so the ceiling that applies to real data is the one measured with random operands
 * (Sec. 4 of the paper reports timings on its own hardware only; rooflines here are measured,
 * not quoted). */
int w2l_probe_mfma(float *out, int blocks, int iters, int random_operands, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* W2L_H */
