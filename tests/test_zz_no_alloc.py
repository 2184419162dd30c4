"""GPU test of ec_decode_score_step_static (the entry point that allocates nothing): two calls in a row through
the C ABI, the second with a smaller input, each compared with ec_decode_score_step on a caller workspace."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2407_18121_amd import binding as ec
from util import quantize, to_dev

pytestmark = pytest.mark.gpu


def _inputs(B, H, G, D, cap, n, dtype, seed):
    rng = np.random.default_rng(seed)
    kc = np.zeros((B, H, cap, D), np.float32)
    vc = np.zeros((B, H, cap, D), np.float32)
    kc[:, :, :n] = quantize(rng.standard_normal((B, H, n, D)) * 1.5, dtype)
    vc[:, :, :n] = quantize(rng.standard_normal((B, H, n, D)), dtype)
    q, kn, vn = (quantize(rng.standard_normal((B, H, D)), dtype) for _ in range(3))
    freq = rng.random((B, G, cap)).astype(np.float32)
    pos = np.tile(np.arange(cap, dtype=np.int32), (B, G, 1))
    return q, kn, vn, kc, vc, pos, freq


def _run(static, B, H, G, D, cap, n, dtype, seed):
    """One call through the raw C ABI; returns (out, k_cache, v_cache, pos, freq) as host arrays."""
    lib = ec.load()
    q, kn, vn, kc, vc, pos, freq = _inputs(B, H, G, D, cap, n, dtype, seed)
    dq, dkn, dvn, dkc, dvc = (to_dev(x, dtype) for x in (q, kn, vn, kc, vc))
    dpos, dfreq = torch.from_numpy(pos).cuda(), torch.from_numpy(freq).cuda()
    out = torch.full((B, H, D), float("nan"), dtype=dkc.dtype, device="cuda")
    dtc = ec.dtype_code(dkc)
    s = torch.cuda.current_stream().cuda_stream
    head = (dq.data_ptr(), dkn.data_ptr(), dvn.data_ptr(), dkc.data_ptr(), dvc.data_ptr(), dpos.data_ptr(),
            dfreq.data_ptr(), B, H, G, D, cap, n, 4242, 1.0 / np.sqrt(D), dtc, out.data_ptr())
    if static:
        rc = lib.ec_decode_score_step_static(*head, s)
    else:
        ws = ec.new_workspace(ec.EC_FN_DECODE_SCORE_STEP, B, H, cap, D, dtc)
        rc = lib.ec_decode_score_step(*head, ws.data_ptr(), ws.numel(), s)
    assert rc == ec.EC_OK, ec.status_string(rc)
    torch.cuda.synchronize()
    return tuple(t.float().cpu().numpy() if t.is_floating_point() else t.cpu().numpy()
                 for t in (out, dkc, dvc, dpos, dfreq))


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_static_scratch_matches_caller_workspace_twice_in_a_row(dtype, D):
    # second call smaller than the first: whatever the first left in the shared array must not matter
    for (B, H, G, cap, n, seed) in ((3, 8, 1, 700, 650, 1), (2, 4, 4, 300, 37, 2)):
        ref = _run(False, B, H, G, D, cap, n, dtype, seed)
        got = _run(True, B, H, G, D, cap, n, dtype, seed)
        for name, a, b in zip(("out", "k_cache", "v_cache", "pos", "freq"), got, ref):
            assert np.isfinite(a).all(), name
            np.testing.assert_array_equal(a, b, err_msg=name)   # same kernels, same order: bit for bit


def test_static_scratch_rejects_shapes_beyond_its_size():
    lib = ec.load()
    one = ctypes.c_void_p(256)   # never dereferenced: the size check fails first
    B, H, cap = 64, 64, 4096     # 4*B*H*(cap+2) = 67 MB > 4 MiB
    assert lib.ec_decode_score_step_static(one, one, one, one, one, None, one, B, H, 1, 128, cap, 10, 0, 0.1,
                                           ec.EC_BF16, one, None) == ec.EC_EWORKSPACE
    assert lib.ec_decode_score_step_static(one, one, one, one, one, None, one, 1, 1, 1, 96, 8, 3, 0, 0.1,
                                           ec.EC_BF16, one, None) == ec.EC_EUNSUPPORTED
