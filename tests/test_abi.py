"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol that
include/w2l.h declares, and rejects bad arguments on the host before launching anything."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.environ.get("W2L_LIB") or os.path.join(ROOT, "paper_1812_07625_amd", "libw2l.so")


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "w2l.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(w2l_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libw2l.so is not built: run `python -m paper_1812_07625_amd.build`")
    return C.CDLL(LIB)


def test_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), "missing export %s" % n


def test_binding_names_match_header():
    import paper_1812_07625_amd as P
    for n in declared_symbols():
        assert hasattr(P, n), "binding lacks %s" % n


def test_status_strings(lib):
    lib.w2l_status_str.restype = C.c_char_p
    seen = set()
    for s in range(0, -8, -1):
        seen.add(lib.w2l_status_str(s))
    assert len(seen) == 8
    assert lib.w2l_version() >= 100


def test_host_side_argument_checks():
    import paper_1812_07625_amd as P
    r = P.raw
    NULL, OK = None, 0
    fake = 0x1000  # never dereferenced: checks fail before any launch
    assert r.w2l_conv1d_fwd(NULL, fake, NULL, fake, 1, 8, 8, 8, 3, 1, 0, 0, NULL, 0, NULL) == -1
    assert r.w2l_conv1d_fwd(fake, fake, NULL, fake, 1, 8, 8, 8, 4, 1, 0, 0, NULL, 0, NULL) == -2  # even k
    assert r.w2l_conv1d_fwd(fake, fake, NULL, fake, 0, 8, 8, 8, 3, 1, 0, 0, NULL, 0, NULL) == -2
    assert r.w2l_conv1d_fwd(fake, fake, NULL, fake, 1, 8, 8, 8, 3, 0, 0, 0, NULL, 0, NULL) == -2
    assert r.w2l_conv1d_fwd(fake, fake, NULL, fake, 1, 8, 8, 8, 3, 1, 7, 0, NULL, 0, NULL) == -3
    assert r.w2l_conv1d_fwd(fake, fake, NULL, fake, 1, 8, 8, 8, 3, 1, 0, 1, NULL, 0, NULL) == -3  # f32 in, bf16 out
    assert r.w2l_conv1d_fwd(fake + 4, fake, NULL, fake, 1, 8, 8, 8, 3, 1, 0, 0, NULL, 0, NULL) == -4
    assert r.w2l_conv1d_bwd_data(fake, NULL, fake, 1, 8, 8, 8, 3, 1, 0, 0, NULL, 0, NULL) == -1
    assert r.w2l_conv1d_bwd_weight(fake, fake, fake, NULL, 1, 8, 8, 8, 3, 1, 0, 0, 0, NULL, 0, NULL) == -5
    assert r.w2l_conv1d_bwd_weight_workspace_bytes(1, 8, 8, 8, 3, 1, 0) > 0
    assert r.w2l_glu_fwd(fake, fake, 4, 7, 0, NULL) == -2  # odd channel count
    assert r.w2l_glu_bwd(fake, NULL, fake, 4, 8, 0, NULL) == -1
    assert r.w2l_logsoftmax_fwd(fake, fake, 4, 5000, 0, NULL) == -2
    assert r.w2l_logsoftmax_bwd(fake, fake, fake, 0, 5, NULL) == -2
    assert r.w2l_ctc_fwd_bwd(fake, 0, fake, fake, fake, fake, fake, 2, 10, 5, 3, 5, 1.0, fake, 1 << 30, NULL) == -2
    assert r.w2l_ctc_fwd_bwd(fake, 0, fake, fake, fake, fake, fake, 2, 10, 5, 3, 0, 1.0, NULL, 0, NULL) == -5
    assert r.w2l_ctc_fwd_bwd(fake, 0, fake, fake, fake, fake, fake, 2, 10, 5, 3, 0, 1.0, 0x1100, 16, NULL) == -5
    assert r.w2l_ctc_workspace_bytes(2, 10, 5, 3) >= 2 * 2 * 10 * 7 * 8
    # size limits: frames (integer state exponents), labels, classes
    assert r.w2l_ctc_fwd_bwd(fake, 0, fake, fake, fake, fake, fake, 2, 8193, 5, 3, 0, 1.0, 0x1100, 1 << 40, NULL) == -2
    assert r.w2l_ctc_fwd_bwd(fake, 0, fake, fake, fake, fake, fake, 2, 10, 5, 3001, 0, 1.0, 0x1100, 1 << 40, NULL) == -2
    assert r.w2l_ctc_fwd_bwd(fake, 0, fake, fake, fake, fake, fake, 2, 10, 4097, 3, 0, 1.0, 0x1100, 1 << 40, NULL) == -2


def test_ctc_host_validation():
    import paper_1812_07625_amd as P
    t = np.array([[1, 2, 3], [4, 4, 0]], np.int32)
    assert P.w2l_ctc_check_targets_host(t, [10, 10], [3, 2], 10, 5) == 0
    assert P.w2l_ctc_check_targets_host(t, [10, 10], [3, 3], 10, 5) == -6   # label 0 = blank
    assert P.w2l_ctc_check_targets_host(t, [10, 11], [3, 2], 10, 5) == -6   # in_len > Tp
    assert P.w2l_ctc_check_targets_host(t, [10, 10], [4, 2], 10, 5) == -6   # tgt_len > Lmax
    assert P.w2l_ctc_check_targets_host(t, [10, 10], [3, 2], 10, 4) == -6   # label >= C


def test_train_step_plan_checks():
    import paper_1812_07625_amd as P
    import workloads as W
    lay = W.layers_105m()
    n = P.w2l_train_step_workspace_bytes(lay, 8, 1500, 150, P.W2L_BF16)
    assert n > 8 * 750 * 1536 * 2 * 9
    bad = [dict(l) for l in lay]
    bad[3]["cin"] = 700   # does not match the previous layer's output channels
    assert P.w2l_train_step_workspace_bytes(bad, 8, 1500, 150, P.W2L_BF16) == 0
    bad = [dict(l) for l in lay]
    bad[-1]["glu"] = 1
    assert P.w2l_train_step_workspace_bytes(bad, 8, 1500, 150, P.W2L_BF16) == 0


def test_host_side_argument_checks_of_the_widened_rows():
    """ASG, log-mel and the optimiser step reject bad arguments before any launch (no GPU needed)."""
    import paper_1812_07625_amd as P
    r = P.raw
    NULL = None
    fake = 0x1000
    ws = 0x1100  # 256-byte aligned, never dereferenced
    # ASG: B, Tp, C, Lmax
    assert r.w2l_asg_fwd_bwd(fake, NULL, fake, fake, fake, fake, fake, fake, 2, 10, 5, 3, 1.0, ws, 1 << 30, NULL) == -1
    assert r.w2l_asg_fwd_bwd(fake, fake, fake, fake, fake, fake, fake, NULL, 2, 10, 65, 3, 1.0, ws, 1 << 30, NULL) == -2  # C > 64
    assert r.w2l_asg_fwd_bwd(fake, fake, fake, fake, fake, fake, fake, NULL, 2, 10, 5, 3001, 1.0, ws, 1 << 30, NULL) == -2
    assert r.w2l_asg_fwd_bwd(fake + 4, fake, fake, fake, fake, fake, fake, NULL, 2, 10, 5, 3, 1.0, ws, 1 << 30, NULL) == -4
    assert r.w2l_asg_fwd_bwd(fake, fake, fake, fake, fake, fake, fake, NULL, 2, 10, 5, 3, 1.0, NULL, 0, NULL) == -5
    assert r.w2l_asg_fwd_bwd(fake, fake, fake, fake, fake, fake, fake, NULL, 2, 10, 5, 3, 1.0, ws, 64, NULL) == -5
    assert r.w2l_asg_workspace_bytes(2, 10, 5, 3) > 4 * 2 * 11 * 7 * 4
    assert r.w2l_asg_workspace_bytes(2, 10, 65, 3) == 0
    t = np.array([[1, 2, 3], [4, 4, 0]], np.int32)
    assert P.w2l_asg_check_targets_host(t, [10, 10], [3, 3], 10, 5) == 0      # label 0 and equal neighbours are fine
    assert P.w2l_asg_check_targets_host(t, [10, 10], [3, 2], 10, 4) == -6     # label >= C
    assert P.w2l_asg_check_targets_host(t, [10, 11], [3, 2], 10, 5) == -6
    # log-mel: B, Nmax, Tmax, n_mels, sample_rate, win, hop, nfft, fmin, fmax, floor, dtype
    ok = (2, 4000, 20, 40, 16000, 400, 160, 512, 0.0, 8000.0, 1e-10, 0)
    assert r.w2l_logmel_fwd(NULL, fake, fake, fake, *ok, NULL) == -1
    for pos, val in ((7, 500), (7, 2048), (5, 600), (3, 256), (9, 9000.0), (8, 8000.0), (10, 0.0), (6, 0)):
        bad = list(ok)
        bad[pos] = val
        assert r.w2l_logmel_fwd(fake, fake, fake, fake, *bad, NULL) == -2, (pos, val)
    bad = list(ok)
    bad[11] = 5
    assert r.w2l_logmel_fwd(fake, fake, fake, fake, *bad, NULL) == -3
    assert r.w2l_logmel_num_frames(400, 400, 160) == 1 and r.w2l_logmel_num_frames(399, 400, 160) == 0
    # optimiser step
    assert r.w2l_sgd_momentum_step(fake, NULL, fake, NULL, 16, 0.1, 0.9, 0.0, NULL) == -1
    assert r.w2l_sgd_momentum_step(fake, fake, fake, NULL, -1, 0.1, 0.9, 0.0, NULL) == -2
    assert r.w2l_sgd_momentum_step(fake + 4, fake, fake, NULL, 16, 0.1, 0.9, 0.0, NULL) == -4
    # train step with ASG: class count and missing transitions
    lay = [dict(k=3, stride=1, cin=8, cout=16, glu=1), dict(k=1, stride=1, cin=8, cout=12, glu=0)]
    assert P.w2l_train_step_asg_workspace_bytes(lay, 2, 20, 4, P.W2L_F32) > 0
    lay[-1]["cout"] = 70
    assert P.w2l_train_step_asg_workspace_bytes(lay, 2, 20, 4, P.W2L_F32) == 0
