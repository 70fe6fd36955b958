"""GPU parity of the device-tuned path (hinm_prepare + hinm_spmm_prepared) against the CPU oracle,
and of the prepared buffer against the canonical arrays it re-orders."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu

OUT_F32, RELU = 2, 1
VARIANTS = [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 13, 14, 16, 17, 15]   # 13, 14, 16, 17 = 32-column waves; 15 = LDS-resident panel kernel (small K only)


def _ulp_bf16(y):
    e = np.floor(np.log2(np.maximum(np.abs(y), 2.0 ** -14)))
    return np.exp2(e - 7)


def _unswizzle(buf: np.ndarray, M, K, V, Kv):
    """Decode the prepared buffer (layout documented in csrc/prepared_layout.h) back into the
    canonical arrays plus the gather table and output rows."""
    T, RB = M // V, V // 32
    Kp = (Kv + 63) // 64 * 64
    S = Kp // 64
    al = lambda x: (x + 255) // 256 * 256
    a_bytes = T * S * RB * 2304
    g_off = al(a_bytes)
    o_off = g_off + al(T * Kp * 4)
    z_off = o_off + al(M * 4)
    blocks = buf[:a_bytes].reshape(T, S, RB, 2304)
    vals_u16 = blocks[..., :2048].copy().view(np.uint16).reshape(T, S, RB, 2, 64, 8)
    idx_u32 = blocks[..., 2048:].copy().view(np.uint32).reshape(T, S, RB, 64)
    G = Kp // 4
    vals = np.zeros((M, G * 2), dtype=np.uint16)
    nib = np.zeros((M, G), dtype=np.uint8)
    for lane in range(64):
        i, qa = lane % 32, lane // 32
        for sub in range(2):
            for k in range(4):
                # group 16 s + 8 sub + 4 qa + k of row 32 rb + i
                for s in range(S):
                    g = 16 * s + 8 * sub + 4 * qa + k
                    rows = (np.arange(T)[:, None] * V + 32 * np.arange(RB)[None, :] + i).reshape(-1)
                    vals[rows, 2 * g] = vals_u16[:, s, :, sub, lane, 2 * k].reshape(-1)
                    vals[rows, 2 * g + 1] = vals_u16[:, s, :, sub, lane, 2 * k + 1].reshape(-1)
                    nib[rows, g] = ((idx_u32[:, s, :, lane] >> (16 * sub + 4 * k)) & 0xF).reshape(-1)
    gather = buf[g_off:g_off + T * Kp * 4].copy().view(np.int32).reshape(T, Kp)
    out_rows = buf[o_off:o_off + M * 4].copy().view(np.int32)
    zeros = buf[z_off:z_off + 1024]
    panel = buf[z_off + 1024:z_off + 1024 + T * Kp * 4].copy().view(np.uint32).reshape(T, Kp)
    K8 = (K + 7) // 8 * 8
    g = gather.astype(np.int64)
    want_panel = np.where(g >= 0, (g << 7) | ((g & 2) << 5), K8 << 7).astype(np.uint32)
    assert np.array_equal(panel, want_panel), "LDS-address form of the gather table"
    return vals, nib, gather, out_rows, zeros


@pytest.mark.parametrize("M,K,V,Kv,dtype", [(128, 256, 32, 128, "f16"), (256, 320, 128, 200, "bf16"),
                                            (192, 256, 96, 64, "f16")])
def test_prepared_buffer_is_a_reordering(M, K, V, Kv, dtype):
    from tests import gpu_util as gu
    case = synth.small_case(M, K, V, Kv, 8, dtype, 80)
    vals, nm, vec = orc.pack(case.weights(), dtype, V, Kv)
    p = gu.upload_packed(M, K, V, Kv, dtype, vals, nm, vec)
    pin, pout = case.pi_in(), case.pi_out()
    pr = gu.gpu_prepare(p, pin, pout)
    v2, nib, gather, out_rows, zeros = _unswizzle(pr.buf.cpu().numpy(), M, K, V, Kv)
    G = Kv // 4
    assert np.array_equal(v2[:, :2 * G], vals)
    assert np.all(v2[:, 2 * G:] == 0)
    want_nib = np.stack([nm & 0xF, nm >> 4], axis=-1).reshape(M, G)
    assert np.array_equal(nib[:, :G], want_nib)
    assert np.all(nib[:, G:] == 0x4)
    assert np.array_equal(gather[:, :Kv], pin[vec])
    assert np.all(gather[:, Kv:] == -1)
    assert np.array_equal(out_rows, pout)
    assert np.all(zeros == 0)
    pr = gu.gpu_prepare(p, None, None)
    _, _, gather, out_rows, _ = _unswizzle(pr.buf.cpu().numpy(), M, K, V, Kv)
    assert np.array_equal(gather[:, :Kv], vec) and np.array_equal(out_rows, np.arange(M))


def _check(case, N, variants, relu=False, identity=False):
    from tests import gpu_util as gu
    vals, nm, vec = orc.pack(case.weights(), case.dtype, case.V, case.Kv)
    Wh = orc.unpack_fast(vals, nm, vec, case.M, case.K, case.V)
    Xb = case.activations(N)
    pin = None if identity else case.pi_in()
    pout = None if identity else case.pi_out()
    Y_acc = orc.product(Wh, Xb, case.dtype, pin, pout, relu=relu).astype(np.float64)
    p = gu.upload_packed(case.M, case.K, case.V, case.Kv, case.dtype, vals, nm, vec)
    pr = gu.gpu_prepare(p, pin, pout)
    f = RELU if relu else 0
    import paper_2407_20496_amd as hinm
    for v in variants:
        try:
            got32 = gu.gpu_spmm_prepared(pr, Xb, f | OUT_F32, variant=v).astype(np.float64)
        except hinm.HinmError as err:
            # the panel kernel refuses shapes whose panel does not fit in LDS; nothing else may refuse
            assert v == 15 and err.status == 5 and (((case.K + 7) // 8 * 8 + 8) * 128 + 8 * 32 * 144 > 160 * 1024 or N <= 32)
            continue
        gu.check_close(got32, Y_acc, what=f"{case.name} variant {v} fp32")
        got = gu.gpu_spmm_prepared(pr, Xb, f, variant=v)
        assert np.array_equal(got, orc.round_to_storage(got32.astype(np.float32), case.dtype)), f"variant {v}"
        if case.dtype == "f16":
            gu.check_close(orc.decode(got, "f16"), Y_acc, what=f"{case.name} variant {v} fp16")
        else:
            want = orc.decode(orc.round_to_storage(Y_acc.astype(np.float32), "bf16"), "bf16")
            gotd = orc.decode(got, "bf16")
            assert np.all(np.abs(gotd - want) <= np.maximum(1e-2, _ulp_bf16(want)))
            gu.check_close(gotd, want, max_abs=np.inf, what=f"{case.name} variant {v} bf16")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M,K,V,Kv,N", [
    (128, 256, 32, 128, 37),
    (128, 320, 64, 160, 300),     # ragged column tail inside the second 256-column block
    (384, 512, 128, 256, 520),    # ragged tail past one 512-column block
    (192, 256, 96, 64, 40),
    (128, 512, 64, 200, 72),      # Kv % 64 != 0: padded kept columns
    (256, 1024, 128, 704, 256),   # 11 steps: odd number of 64-column steps
])
def test_prepared_small_all_variants(M, K, V, Kv, N, dtype):
    _check(synth.small_case(M, K, V, Kv, N, dtype, 81), N, VARIANTS)


@pytest.mark.parametrize("M,K,V,Kv,N,dtype", [
    (2752, 1152, 32, 576, 2048, "f16"),      # 86 tiles x 4 wide blocks: 64 tiles in wide blocks, 22 in narrow ones
    (11008, 1152, 128, 576, 2048, "bf16"),   # the same split with 128-row tiles
    (5504, 1280, 64, 640, 1500, "f16"),      # 86 tiles x 3 wide blocks (ragged last block): 85 + 1
])
def test_prepared_remainder_tiles_in_a_second_launch(M, K, V, Kv, N, dtype):
    """Layers whose wide blocks make whole rounds plus a small remainder are launched in two parts."""
    _check(synth.small_case(M, K, V, Kv, N, dtype, 83), N, [0, 3, 16])


def test_prepared_relu_identity():
    case = synth.small_case(128, 256, 64, 128, 72, "f16", 82)
    _check(case, 72, [0, 2, 3], relu=True)
    _check(case, 72, [0, 2, 3], identity=True)


def test_prepared_c2_full():
    c = synth.c2()
    _check(c, c.N, [0, 1, 3, 8, 15])


def test_prepared_panel_kernel_edges():
    # K not a multiple of 8, ragged N, padded kept columns, one tile per wave and fewer tiles than waves
    _check(synth.small_case(64, 100, 32, 40, 70, "f16", 85), 70, [15])
    _check(synth.small_case(96, 1000, 32, 504, 130, "bf16", 86), 130, [15], relu=True)
    _check(synth.small_case(64, 512, 64, 256, 64, "f16", 87), 64, [15], identity=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M,K,V,Kv,N", [
    (128, 256, 32, 128, 1),
    (256, 1024, 128, 704, 16),    # several workgroups per tile, odd number of steps
    (128, 2048, 64, 1032, 3),     # padded kept columns (Kv % 64 != 0)
    (192, 512, 96, 256, 17),
    (256, 4096, 128, 2048, 32),
    (128, 512, 128, 64, 8),       # a single step: no split
    (64, 4224, 32, 2200, 1),      # one column, more than 32 steps: the input vector is staged in LDS; padded steps
    (64, 4220, 32, 2112, 1),      # K % 8 != 0: same shape class without staging
    (32, 12288, 32, 8192, 1),     # 128 steps over 16 waves: the 16-row kernel stages the input vector as well
])
def test_prepared_few_columns(M, K, V, Kv, N, dtype):
    # 0 = by shape, 11 = 16-row workgroups (16x16x64 form), 12 = 32-row workgroups (32x32x32 form)
    _check(synth.small_case(M, K, V, Kv, N, dtype, 83), N, [0, 11, 12])


@pytest.mark.parametrize("M,K,V,Kv,N,dtype", [
    (128, 320, 64, 160, 300, "f16"),      # many column blocks, ragged tail, padded kept columns
    (192, 256, 96, 64, 40, "bf16"),       # a single step; 96-row tiles: three 32-row blocks
    (256, 8192, 128, 4416, 16, "bf16"),   # 69 steps: sixteen waves with more than one batch
    (8192, 256, 64, 128, 13, "f16"),      # 256 row blocks of 32: both halves of a block in one workgroup
    # many workgroups: fewer waves each, several batches per wave
    (4096, 1024, 128, 512, 136, "bf16"),  # 2304 workgroups: one wave walks all 8 steps
    (2048, 2304, 128, 1152, 72, "f16"),   # 640 workgroups: two waves, 9 steps each
    (8192, 512, 64, 384, 88, "bf16"),     # 1536 workgroups of 32 rows: one wave, 6 steps in two batches
    (512, 4608, 32, 2304, 392, "f16"),    # 36 steps, two column blocks per workgroup, ragged last block of 8
    (4096, 2048, 128, 1024, 72, "bf16"),  # 64-row workgroups with two column blocks; the last pair holds 8 columns
    (4096, 2048, 128, 1024, 200, "f16"),  # 64-row workgroups with four column blocks; the last four hold 8 columns
    (2048, 2304, 32, 1152, 136, "bf16"),  # 32-row tiles, four column blocks, 18 steps
])
def test_prepared_sixteen_row_kernel_beyond_few_columns(M, K, V, Kv, N, dtype):
    _check(synth.small_case(M, K, V, Kv, N, dtype, 88), N, [11])
    _check(synth.small_case(M, K, V, Kv, N, dtype, 89), N, [11], relu=True, identity=True)


def test_prepared_few_columns_on_a_large_layer_and_garbage_in_the_padding():
    """Up to 64 columns go to the 16-row kernel when the layer is large; columns of X beyond N (inside the
    leading dimension) may hold anything."""
    import torch
    from tests import gpu_util as gu
    case = synth.small_case(4096, 2048, 128, 1024, 40, "f16", 90)
    _check(case, 40, [0, 11])
    _padding_may_hold_anything(synth.small_case(256, 1024, 64, 512, 19, "bf16", 91), 19, 24, (0, 11, 12))
    # two column blocks per workgroup: the second pair covers columns 32..47 of the row and nothing beyond
    _padding_may_hold_anything(synth.small_case(2048, 2304, 128, 1152, 40, "f16", 92), 40, 48, (0, 11))


def _padding_may_hold_anything(case, N, ld, variants):
    from tests import gpu_util as gu
    p = gu.gpu_pack(case.weights(), case.dtype, case.V, case.Kv)
    pr = gu.gpu_prepare(p, case.pi_in(), case.pi_out())
    Xb = case.activations(N)
    Xp = np.full((case.K, ld), 0x7FC0, dtype=np.uint16)     # NaN in every padding column
    Xp[:, :N] = Xb
    for variant in variants:
        want = gu.gpu_spmm_prepared(pr, Xb, variant=variant, ldx=ld, ldy=ld)
        got = gu.gpu_spmm_prepared(pr, Xb, variant=variant, ldx=ld, ldy=ld, X_dev=gu.dev_bits(Xp))
        assert np.array_equal(got, want), f"variant {variant}"


@pytest.mark.parametrize("M,K,V,Kv,dtype", [
    (256, 512, 64, 256, "f16"),       # four steps: one wave per step
    (384, 1000, 128, 504, "bf16"),    # K % 32 != 0, Kv % 64 != 0: clamped copies, padded kept columns
    (128, 4096, 128, 2048, "f16"),    # 32 steps: the largest input that fits beside eight slabs
    (192, 2048, 64, 1024, "bf16"),
    (128, 256, 64, 128, "f16"),       # two steps, 8 KB of input rows: the waves' partial tiles (16 KB) need more LDS
    (128, 640, 128, 576, "bf16"),     # nine steps over four waves, 20 KB of input rows
])
def test_prepared_sixteen_columns_input_resident_in_lds(M, K, V, Kv, dtype):
    case = synth.small_case(M, K, V, Kv, 16, dtype, 86)
    _check(case, 16, [0, 11, 19])
    _check(case, 16, [19], relu=True)
    _check(case, 16, [19], identity=True)


def test_prepared_input_resident_variant_refuses_what_it_cannot_hold():
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    for (M, K, V, Kv, N) in [(128, 8192, 128, 4096, 16),    # 256 KB of input rows
                             (128, 512, 32, 256, 16),       # V % 64 != 0
                             (128, 512, 64, 256, 8)]:       # not 16 columns
        case = synth.small_case(M, K, V, Kv, N, "f16", 87)
        p = gu.gpu_pack(case.weights(), "f16", V, Kv)
        pr = gu.gpu_prepare(p, case.pi_in(), case.pi_out())
        with pytest.raises(hinm.HinmError) as err:
            gu.gpu_spmm_prepared(pr, case.activations(N), variant=19)
        assert err.value.status == 5


def test_prepared_few_columns_repeatable_and_needs_no_workspace():
    # partial tiles are added in a fixed order: repeated calls give identical bits
    import torch
    from tests import gpu_util as gu
    import paper_2407_20496_amd as hinm
    case = synth.small_case(256, 2048, 128, 1024, 16, "bf16", 84)
    vals, nm, vec = orc.pack(case.weights(), "bf16", 128, 1024)
    p = gu.upload_packed(256, 2048, 128, 1024, "bf16", vals, nm, vec)
    pr = gu.gpu_prepare(p, case.pi_in(), case.pi_out())
    assert hinm.hinm_spmm_prepared_workspace(256, 2048, 128, 1024, "bf16", 16) == 0
    Xd = gu.dev_bits(case.activations())
    outs = []
    for _ in range(3):
        Y = torch.zeros((256, 16), dtype=torch.int16, device=gu.DEV)
        hinm.hinm_spmm_prepared(256, 2048, 128, 1024, "bf16", 16, pr.buf, Xd, 16, Y, 16, 0, None, 0)
        torch.cuda.synchronize()
        outs.append(gu.host_bits(Y))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    Wh = orc.unpack_fast(vals, nm, vec, 256, 2048, 128)
    want = orc.product(Wh, case.activations(), "bf16", case.pi_in(), case.pi_out()).astype(np.float64)
    got = orc.decode(outs[0], "bf16")
    assert np.all(np.abs(got - want) <= np.maximum(1e-2, _ulp_bf16(want)))


@pytest.mark.parametrize("idx", [0, 1, 3, 4, 6, 7, 9, 10])
def test_prepared_c3_decode_full(idx):
    c = synth.c3_cases()[idx]
    assert c.N in (1, 16)
    _check(c, c.N, [0])


def test_tile_kernel_parts_run_and_store_nothing():
    """The measurement launches (copy stream alone, LDS reads and MFMAs alone) finish, leave X and the prepared
    layer as they were, and the product launched afterwards on the same buffers is still right."""
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    shapes = [(4096, 1024, 128, 512, 1100, "bf16"), (1024, 2048, 64, 1024, 1032, "f16")]   # both run on the tile kernel
    for (M, K, V, Kv, N, dtype) in shapes:
        ld = (N + 7) // 8 * 8
        assert "spmm_tile_prepared_kernel" in hinm.hinm_spmm_prepared_plan(M, K, V, Kv, dtype, N, ld, ld, 0)[0]
        case = synth.small_case(M, K, V, Kv, N, dtype, 77)
        vals, nm, vec = orc.pack(case.weights(), case.dtype, V, Kv)
        p = gu.upload_packed(M, K, V, Kv, dtype, vals, nm, vec)
        pr = gu.gpu_prepare(p, case.pi_in(), case.pi_out())
        prep = pr.buf
        ld = (N + 7) // 8 * 8
        Xh = np.zeros((K, ld), dtype=np.uint16)
        Xh[:, :N] = case.activations(N)
        X = torch.from_numpy(Xh.view(np.int16)).cuda()
        before_x, before_p = X.clone(), prep.clone()
        for part in (1, 2):
            hinm.hinm_calib_tile_part(M, K, V, Kv, dtype, N, prep, X, ld, part)
        torch.cuda.synchronize()
        assert torch.equal(X, before_x) and torch.equal(prep, before_p)
    with pytest.raises(hinm.HinmError):     # a shape served by another kernel has no tile-kernel parts
        hinm.hinm_calib_tile_part(256, 512, 64, 256, "f16", 520, prep, X, 520, 1)
    _check(synth.small_case(1024, 2048, 64, 1024, 1032, "f16", 77), 1032, [0])
