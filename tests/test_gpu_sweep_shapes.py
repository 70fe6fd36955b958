"""GPU parity on the layer shapes of the latency sweep (`bench.py --workload sweep-bert / sweep-resnet`;
Section 5.3 and the V = 32 convolution setting of Section 5.1.1): every vector size and vector sparsity the
sweep times, full size, through the kernel the library picks by shape.  Packing bit-exact against the
oracle, products on sampled outputs."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu


def _cases():
    out, seen = [], set()
    for which, v_list in (("sweep-bert", (32, 64, 128)), ("sweep-resnet", (32,))):
        for (_, M, K, N) in synth.sweep_layers(which):
            for V in v_list:
                for keep in (2, 4, 8):
                    key = (M, K, N, V, keep)
                    if M % V == 0 and key not in seen:
                        seen.add(key)
                        out.append(key)
    return out


@pytest.mark.parametrize("M,K,N,V,keep", _cases())
def test_sweep_shape(M, K, N, V, keep):
    from tests import gpu_util as gu
    Kv = K // keep
    c = synth.small_case(M, K, V, Kv, N, "f16", 60 + keep)
    Wb, Xb = c.weights(), c.activations()
    p = gu.gpu_pack(Wb, c.dtype, V, Kv)
    vals, nm, vec = orc.pack(Wb, c.dtype, V, Kv)
    for got, want in zip(p.host(), (vals, nm, vec)):
        assert np.array_equal(got, want)
    Wh = orc.unpack_fast(vals, nm, vec, M, K, V)
    pin, pout = c.pi_in(), c.pi_out()
    got = gu.gpu_spmm_prepared(gu.gpu_prepare(p, pin, pout), Xb, 2).astype(np.float64)   # fp32 accumulators
    rng = np.random.default_rng(61)
    rows = rng.choice(M, min(M, 40), replace=False)
    cols = np.unique(np.concatenate([rng.choice(N, 60, replace=False), [0, N - 1]]))
    want = orc.product_entries(Wh, Xb, c.dtype, pin, pout, rows, cols)
    gu.check_close(got[np.asarray(pout)[rows]][:, cols], want, what=f"{M}x{K} N{N} V{V} keep 1/{keep}")
