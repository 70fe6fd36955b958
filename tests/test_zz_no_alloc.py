"""hinm_pack_static (the entry point that allocates nothing: its score workspace is a device array inside
the library) against hinm_pack, through the C ABI, on two calls in a row, the second on a smaller layer."""
import ctypes as C

import numpy as np
import pytest

import hinm_synth as synth

pytestmark = pytest.mark.gpu


def _pack_both(lib, binding, torch, M, K, V, Kv, dtype, salt):
    """Runs hinm_pack and hinm_pack_static on the same W with raw ctypes calls; returns both results."""
    dev = "cuda:0"
    code = 0 if dtype == "f16" else 1
    Wb = synth.small_case(M, K, V, Kv, 8, dtype, salt).weights()
    W = torch.from_numpy(Wb.view(np.int16)).to(dev)
    sh = binding._Shape(M, K, V, Kv, code)
    sizes = [C.c_size_t(0) for _ in range(4)]
    assert lib.hinm_pack_sizes(C.byref(sh), *[C.byref(s) for s in sizes]) == 0
    vb, nb, cb, wb = (int(s.value) for s in sizes)
    out = []
    for static in (False, True):
        vals = torch.full((vb // 2,), 0x7B7B, dtype=torch.int16, device=dev)
        nm = torch.full((nb,), 0xEE, dtype=torch.uint8, device=dev)
        vec = torch.full((cb // 4,), -7, dtype=torch.int32, device=dev)
        if static:
            before = torch.cuda.memory_allocated()
            st = lib.hinm_pack_static(C.byref(sh), W.data_ptr(), vals.data_ptr(), nm.data_ptr(), vec.data_ptr(), None)
            assert torch.cuda.memory_allocated() == before
        else:
            ws = torch.empty(wb, dtype=torch.uint8, device=dev)
            st = lib.hinm_pack(C.byref(sh), W.data_ptr(), vals.data_ptr(), nm.data_ptr(), vec.data_ptr(),
                               ws.data_ptr(), wb, None)
        assert st == 0, st
        torch.cuda.synchronize()
        out.append((vals.cpu().numpy(), nm.cpu().numpy(), vec.cpu().numpy()))
    return out


def test_pack_static_matches_pack_on_two_calls_in_a_row():
    import torch
    import paper_2407_20496_amd as hinm
    from paper_2407_20496_amd import binding
    lib = hinm.load_library()
    # first a layer that uses most of the array (64 tiles x 8192 columns = all 524288 scores), then a smaller one
    # whose scores overwrite only the array's beginning: what the first call left behind must not matter
    for (M, K, V, Kv, dtype, salt) in [(4096, 8192, 64, 4096, "bf16", 70), (384, 1000, 128, 504, "f16", 71)]:
        (v0, n0, c0), (v1, n1, c1) = _pack_both(lib, binding, torch, M, K, V, Kv, dtype, salt)
        assert np.array_equal(c0, c1), "vector index"
        assert np.array_equal(n0, n1), "NM index"
        assert np.array_equal(v0, v1), "stored values"
        assert (c1 >= 0).all()


def test_pack_static_rejects_layers_beyond_its_array():
    import paper_2407_20496_amd as hinm
    from paper_2407_20496_amd import binding
    lib = hinm.load_library()
    fake = 0x1000  # never dereferenced: the size check comes first
    sh = binding._Shape(16384, 16384, 128, 8192, 1)      # 128 tiles x 16384 columns = 4 x the limit
    assert lib.hinm_pack_static(C.byref(sh), fake, fake, fake, fake, None) == 4
    sh = binding._Shape(8192, 8200, 128, 4096, 1)        # just beyond: 64 x 8200 > 524288
    assert lib.hinm_pack_static(C.byref(sh), fake, fake, fake, fake, None) == 4
    assert hinm.PACK_STATIC_MAX_SCORES == 524288
