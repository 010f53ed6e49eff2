"""mqa_decode_step_noalloc (the entry point for callers that cannot allocate: its partial softmax
states live in a static device buffer inside the library) against mqa_decode_step, on two calls in
a row, the second with a smaller input, and against the float64 oracle."""
import ctypes

import numpy as np
import pytest
import torch

import mqa_inputs as mi
from oracle import mqa_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def m():
    import paper_1911_02150_amd as lib
    lib.load_library()
    return lib


def _noalloc_raw(m, q, K, V, lens, o):
    """Straight through the C ABI: pointers and sizes, nothing else."""
    from paper_1911_02150_amd import binding
    lib = binding.load_library()
    b, h, k = q.shape
    cap, v = V.shape[-2], V.shape[-1]
    vp = ctypes.c_void_p
    return lib.mqa_decode_step_noalloc(vp(q.data_ptr()), vp(K.data_ptr()), vp(V.data_ptr()), vp(lens.data_ptr()),
                                       vp(o.data_ptr()), b, h, cap, k, v, m.MQA_BF16, ctypes.c_float(1.0),
                                       vp(torch.cuda.current_stream().cuda_stream))


def _case(seed, b, h, cap, lens):
    c = mi.random_case(seed, b, h, cap, 128, 128, cache="bf16", lens=lens)
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = mi.bits_to_torch_bf16(c["K"]).to(DEV), mi.bits_to_torch_bf16(c["V"]).to(DEV)
    dl = torch.from_numpy(c["lens"]).to(DEV)
    ref = orc.mqa_decode(c["q"], mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"])
    return q, K, V, dl, ref


def test_noalloc_matches_the_workspace_call_twice_in_a_row(m):
    # first call: 6 sequences x 4000 positions -> the heuristics split every sequence into many ranges,
    # so the static buffer holds partial states; second call: fewer, shorter sequences (fewer ranges),
    # which must not see anything the first call left behind
    # (the first call on a device looks up the buffer's address, at which point the runtime materialises the
    # library's device variables: that one-time set-up is done here, before memory is watched)
    q, K, V, dl, _ = _case(69, 2, 8, 64, "full")
    assert _noalloc_raw(m, q, K, V, dl, torch.empty((2, 8, 128), dtype=torch.float32, device=DEV)) == 0
    torch.cuda.synchronize()
    for seed, b, h, cap, lens in ((70, 6, 32, 4000, "ragged"), (71, 3, 8, 700, [700, 1, 333])):
        q, K, V, dl, ref = _case(seed, b, h, cap, lens)
        assert m.mqa_decode_num_splits(b, h, cap, 128, 128, m.MQA_BF16) > 1
        assert m.mqa_decode_workspace_bytes_default(b, h, cap, 128, 128, m.MQA_BF16) > 0
        want = m.mqa_decode_step(q, K, V, dl)
        torch.cuda.synchronize()
        o = torch.full_like(want, float("nan"))
        torch.cuda.synchronize()
        allocated, free_on_device = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
        rc = _noalloc_raw(m, q, K, V, dl, o)
        torch.cuda.synchronize()
        assert rc == 0, m.status_string(rc)
        # nothing was allocated: neither through torch nor behind its back (the device's free memory is unchanged)
        assert torch.cuda.memory_allocated() == allocated and torch.cuda.mem_get_info()[0] == free_on_device
        assert torch.equal(o, want), "static-buffer call differs from the workspace call"
        err = float(np.max(np.abs(o.cpu().numpy().astype(np.float64) - ref)))
        assert err <= 2e-2 and err <= 1e-2 * float(np.max(np.abs(ref)))


def test_noalloc_single_range_and_ordered_batch(m):
    # one range per sequence (nothing in the buffer but the length schedule), through the binding
    q, K, V, dl, ref = _case(72, 300, 8, 96, "with_zero")
    o = m.mqa_decode_step_noalloc(q, K, V, dl, torch.empty((300, 8, 128), dtype=torch.float32, device=DEV))
    assert torch.equal(o, m.mqa_decode_step(q, K, V, dl))
    err = float(np.max(np.abs(o.cpu().numpy().astype(np.float64) - ref)))
    assert err <= 2e-2


def test_noalloc_rejects_what_does_not_fit(m):
    """A plan that needs more than the static buffer is refused before anything is enqueued.  (The default
    plans keep the partial states under 4.3 MB for any shape -- about 8192 (row, range) pairs -- so what can
    outgrow the buffer is the length schedule of a very large batch.)"""
    from paper_1911_02150_amd import binding
    lib = binding.load_library()
    b, h, cap = 5_000_000, 1, 32
    assert m.mqa_decode_workspace_bytes_default(b, h, cap, 128, 128, m.MQA_BF16) > (8 << 20)
    vp = ctypes.c_void_p
    A = vp(0x10000)                                # never dereferenced: the size check comes first
    rc = lib.mqa_decode_step_noalloc(A, A, A, A, A, b, h, cap, 128, 128, m.MQA_BF16, ctypes.c_float(1.0), None)
    assert rc == 7 and "static buffer" in m.status_string(rc)
