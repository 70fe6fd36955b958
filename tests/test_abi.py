"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every declared entry point, computes sizes, and rejects bad arguments before
launching anything."""
import ctypes as C
import os
import re

import pytest

import paper_2407_20496_amd as hinm
from paper_2407_20496_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    """Every function declared by a header under include/."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if header.endswith(".h"):
            text = open(os.path.join(inc, header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(hinm_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = hinm.load_library()
    names = declared_functions()
    assert set(names) == set(hinm.exported_symbols())
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    assert hinm.hinm_version() >= 1
    assert hinm.hinm_status_str(0) == "ok"
    for s in range(1, 7):
        assert hinm.hinm_status_str(s) not in ("ok", "unknown status")


def test_pack_sizes():
    v, n, c, w = hinm.hinm_pack_sizes(3072, 768, 64, 384, "f16")
    assert (v, n, c, w) == (3072 * 192 * 2, 3072 * 48, 48 * 384 * 4, 48 * 768 * 8)


@pytest.mark.parametrize("M,K,V,Kv,dtype,status", [
    (256, 256, 17, 128, 0, 2),    # M % V != 0
    (256, 256, 16, 132, 0, 2),    # Kv % 8 != 0
    (256, 256, 16, 264, 0, 2),    # Kv > K
    (0, 256, 16, 128, 0, 2),
    (256, 256, 16, 128, 7, 3),    # dtype
])
def test_shape_errors(M, K, V, Kv, dtype, status):
    lib = hinm.load_library()
    sh = binding._Shape(M, K, V, Kv, dtype)
    out = C.c_size_t(0)
    assert lib.hinm_pack_sizes(C.byref(sh), C.byref(out), None, None, None) == status


def test_null_and_workspace_errors_are_reported_before_any_launch():
    lib = hinm.load_library()
    sh = binding._Shape(256, 256, 16, 128, 0)
    fake = 0x1000  # never dereferenced: validation fails first
    assert lib.hinm_pack(C.byref(sh), None, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.hinm_pack(C.byref(sh), fake, fake, fake, fake, None, 0, None) == 4
    assert lib.hinm_pack(C.byref(sh), fake, fake, fake, fake, fake, 16, None) == 4      # too small
    assert lib.hinm_unpack(C.byref(sh), fake, fake, None, fake, None) == 1
    # ordered pack: same checks as hinm_pack, then the order's alignment and the K limit of its bitmap
    assert lib.hinm_pack_ordered(C.byref(sh), None, fake, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.hinm_pack_ordered(C.byref(sh), fake, fake, fake, fake, fake, None, 0, None) == 4
    assert lib.hinm_pack_ordered(C.byref(sh), fake, fake + 2, fake, fake, fake, fake, 1 << 20, None) == 5
    big = binding._Shape(16, 400000, 16, 8, 0)
    assert lib.hinm_pack_ordered(C.byref(big), fake, fake, fake, fake, fake, fake, 1 << 30, None) == 5
    # scored pack: null rho, misaligned rho; vector-only pack: misaligned vals_v, rho optional (checks go on to
    # the workspace); vector-only product: null, bad N, bad ld, misaligned vals_v, a flag it does not know
    assert lib.hinm_pack_scored(C.byref(sh), fake, None, None, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.hinm_pack_scored(C.byref(sh), fake, fake + 2, None, fake, fake, fake, fake, 1 << 20, None) == 2
    assert lib.hinm_pack_scored(C.byref(sh), fake, fake, None, fake, None, fake, fake, 1 << 20, None) == 1
    assert lib.hinm_pack_vectors(C.byref(sh), fake, None, None, fake + 8, fake, fake, 1 << 20, None) == 2
    assert lib.hinm_pack_vectors(C.byref(sh), fake, None, None, fake, fake, None, 0, None) == 4
    assert lib.hinm_pack_vectors(C.byref(sh), fake, None, None, None, fake, fake, 1 << 20, None) == 1

    def vcall(N=64, vals_v=fake, X=fake, ldx=64, ldy=64, flags=0):
        return lib.hinm_spmm_vectors(C.byref(sh), N, vals_v, fake, None, None, X, ldx, fake, ldy, flags, None)
    assert vcall(X=None) == 1
    assert vcall(N=0) == 2
    assert vcall(ldx=60) == 2
    assert vcall(ldy=68) == 2
    assert vcall(vals_v=fake + 8) == 2
    assert vcall(flags=2 << 16) == 5     # V = 16 here: no tile kernel to pin
    assert vcall(flags=0x100 | 1 << 16) == 5
    assert vcall(flags=0x200) == 5           # HINM_KERNEL_SMFMAC has no meaning for a layer without the 2:4 mask
    # permutation search: neither W nor rho, no samples, bad iteration count, workspace, more than 1024 partitions
    need = C.c_size_t(0)
    assert lib.hinm_icp_sizes(C.byref(sh), C.byref(need)) == 0 and need.value > 0
    assert lib.hinm_icp_search(C.byref(sh), None, None, fake, fake, 1, None, fake, 1 << 30, None) == 1
    assert lib.hinm_icp_search(C.byref(sh), fake, None, fake, None, 1, None, fake, 1 << 30, None) == 1
    assert lib.hinm_icp_search(C.byref(sh), fake, None, fake, fake, -1, None, fake, 1 << 30, None) == 2
    assert lib.hinm_icp_search(C.byref(sh), fake, None, fake, fake, 1, None, fake, 16, None) == 4
    assert lib.hinm_icp_search(C.byref(sh), fake, None, fake, fake, 1, None, fake + 8, 1 << 30, None) == 4
    wide = binding._Shape(16, 8192, 16, 4104, 0)
    assert lib.hinm_icp_sizes(C.byref(wide), C.byref(need)) == 5
    # output-channel search: sample count, nulls, workspace, limits
    assert lib.hinm_ocp_sizes(C.byref(sh), 0, C.byref(need)) == 2
    assert lib.hinm_ocp_sizes(C.byref(sh), 17, C.byref(need)) == 2          # more samples than channels in a tile
    assert lib.hinm_ocp_sizes(C.byref(sh), 4, C.byref(need)) == 0 and need.value > 0
    assert lib.hinm_ocp_search(C.byref(sh), None, None, fake, fake, None, 4, 1, None, fake, 1 << 30, None) == 1
    assert lib.hinm_ocp_search(C.byref(sh), fake, None, None, fake, None, 4, 1, None, fake, 1 << 30, None) == 1
    assert lib.hinm_ocp_search(C.byref(sh), fake, None, fake, fake, None, 4, 1, None, fake, 16, None) == 4
    assert lib.hinm_ocp_search(C.byref(sh), fake, None, fake, fake + 2, None, 4, 1, None, fake, 1 << 30, None) == 2
    many = binding._Shape(32768, 64, 16, 32, 0)                                # 2048 tiles
    assert lib.hinm_ocp_sizes(C.byref(many), 1, C.byref(need)) == 5
    # clustering: the point count limit, rounds, nulls
    assert lib.hinm_ocp_cluster_sizes(C.byref(sh), 4, C.byref(need)) == 0 and need.value > 0
    big_t = binding._Shape(16384, 64, 16, 32, 0)                               # 1024 tiles x 2 samples > 1024 points
    assert lib.hinm_ocp_cluster_sizes(C.byref(big_t), 2, C.byref(need)) == 5
    assert lib.hinm_ocp_cluster(C.byref(sh), fake, None, fake, fake, 4, 0, fake, 1, fake, None, fake, 1 << 30, None) == 2
    assert lib.hinm_ocp_cluster(C.byref(sh), fake, None, fake, fake, 4, 1, None, 1, fake, None, fake, 1 << 30, None) == 1
    assert lib.hinm_ocp_cluster(C.byref(sh), fake, None, fake, fake, 4, 1, fake, 1, fake, None, None, 0, None) == 4
    # spmm: null X, bad N, bad ld, misaligned X, unknown flag, two kernels forced
    args = dict(N=64, vals=fake, nm=fake, vec=fake, X=fake, ldx=64, Y=fake, ldy=64, flags=0)

    def call(**kw):
        a = dict(args, **kw)
        return lib.hinm_spmm(C.byref(sh), a["N"], a["vals"], a["nm"], a["vec"], None, None, a["X"], a["ldx"],
                             a["Y"], a["ldy"], a["flags"], None, 0, None)
    assert call(X=None) == 1
    assert call(N=0) == 2
    assert call(ldx=60) == 2
    assert call(ldx=68) == 2            # not a multiple of 8
    assert call(X=fake + 2) == 2
    assert call(flags=0x8000) == 5
    assert call(flags=0x300) == 5


def test_pack_static_rejects_layers_beyond_its_array_before_touching_the_device():
    lib = hinm.load_library()
    fake = 0x1000
    big = binding._Shape(16384, 16384, 128, 8192, 1)          # 128 tiles x 16384 columns: four times the array
    assert lib.hinm_pack_static(C.byref(big), fake, fake, fake, fake, None) == 4
    edge = binding._Shape(8192, 8200, 128, 4096, 1)           # 64 x 8200 scores: just beyond
    assert lib.hinm_pack_static(C.byref(edge), fake, fake, fake, fake, None) == 4
    ok_shape = binding._Shape(256, 256, 16, 128, 0)
    assert lib.hinm_pack_static(C.byref(ok_shape), None, fake, fake, fake, None) == 1
    assert lib.hinm_pack_static(C.byref(ok_shape), fake, fake + 2, fake, fake, None) == 2
    text = open(os.path.join(ROOT, "include", "hinm.h")).read()
    assert f"#define HINM_PACK_STATIC_MAX_SCORES {hinm.PACK_STATIC_MAX_SCORES}" in text


def test_plan_query_names_the_kernels_without_a_device():
    text, n = hinm.hinm_spmm_prepared_plan(16384, 16384, 128, 8192, "bf16", 8192, 8192, 8192)
    assert n == 1 and text.startswith("spmm_tile_prepared_kernel<") and "NB=512" in text
    text, n = hinm.hinm_spmm_prepared_plan(11008, 4096, 128, 2048, "bf16", 2048, 2048, 2048)
    assert n == 2 and text.count("spmm_tile_prepared_kernel") == 2 and "; " in text   # whole rounds + remainder
    text, n = hinm.hinm_spmm_prepared_plan(3072, 768, 64, 384, "f16", 4096, 4096, 4096)
    assert n == 1 and text.startswith("spmm_panel_prepared_kernel<")
    text, n = hinm.hinm_spmm_prepared_plan(4096, 11008, 128, 5504, "bf16", 1, 1, 1)
    assert n == 1 and text.startswith("spmm_rows16_prepared_kernel<")
    # a pinned kernel that does not fit the shape is refused here exactly as by the product call
    with pytest.raises(hinm.HinmError) as err:
        hinm.hinm_spmm_prepared_plan(128, 8192, 128, 4096, "f16", 16, 16, 16, flags=19 << 16)
    assert err.value.status == 5
    with pytest.raises(hinm.HinmError) as err:
        hinm.hinm_spmm_prepared_plan(256, 256, 16, 128, "f16", 64, 64, 64)       # V = 16: no prepared form
    assert err.value.status == 5


def test_chain_rejects_a_pinned_kernel_that_does_not_fit_before_launching_anything():
    lib = hinm.load_library()
    fake = 0x100000
    ok = binding._Layer(binding._Shape(256, 256, 64, 128, 0), None, None, None, None, None, 0, fake)
    # second layer pins the LDS-resident 16-column kernel (variant 19) at N = 8: unsupported
    bad = binding._Layer(binding._Shape(256, 256, 64, 128, 0), None, None, None, None, None, 19 << 16, fake)
    two = (binding._Layer * 2)(ok, bad)
    assert lib.hinm_chain(2, two, 8, fake, 8, fake, 8, fake, 1 << 20, None) == 5
    # ... and the tile branch at one column
    bad1 = binding._Layer(binding._Shape(256, 256, 64, 128, 0), None, None, None, None, None, 3 << 16, fake)
    two = (binding._Layer * 2)(ok, bad1)
    assert lib.hinm_chain(2, two, 1, fake, 1, fake, 1, fake, 1 << 20, None) == 5


def test_calibration_entry_points_validate_before_launching():
    lib = hinm.load_library()
    fake = 0x100000
    assert lib.hinm_calib_copy(None, fake, 1024, 0, None) == 1
    assert lib.hinm_calib_copy(fake, fake + 4096, 1000, 0, None) == 2          # not a multiple of 16
    assert lib.hinm_calib_copy(fake + 8, fake + 4096, 1024, 0, None) == 2       # misaligned
    assert lib.hinm_calib_fill(None, 1024, 0, None) == 1
    assert lib.hinm_calib_read(fake, 1024, 0, None, None) == 1
    assert lib.hinm_calib_scatter_rows(fake, 64, 256, 256, None, 96, None) == 2   # piece size
    assert lib.hinm_calib_scatter_rows(fake, 64, 96, 96, None, 128, None) == 2    # row bytes not a multiple of the piece
    assert lib.hinm_calib_smfmac(5, 10, fake, None, None) == 3
    assert lib.hinm_calib_smfmac(0, 0, fake, None, None) == 2
    assert lib.hinm_calib_lds_stream(fake, 1000, 0, 1, 1, None) == 2
    assert lib.hinm_calib_lds_stream(fake, 8192, 100, 1, 1, None) == 2
    assert lib.hinm_calib_gather_stream(None, 1 << 20, 16384, 64, 2, 8, 10, 4, None) == 1
    assert lib.hinm_calib_gather_stream(fake, 1 << 20, 16384, 65, 2, 8, 10, 4, None) == 2       # rows x pitch beyond the region
    assert lib.hinm_calib_gather_stream(fake, 1 << 20, 4096, 64, 2, 8, 10, 4, None) == 2        # pitch below 8 KB
    assert lib.hinm_calib_gather_stream(fake, 1 << 20, 16384, 64, 9, 8, 10, 4, None) == 2       # more waves than a workgroup has
    assert lib.hinm_calib_gather_stream(fake, 1 << 20, 16384, 64, 2, 5, 10, 4, None) == 5       # copies in flight: 4, 8 or 16
    # a part of the tile kernel: the same argument checks as the product, then only shapes that kernel serves
    sh = binding._shape(256, 512, 64, 256, "bf16")
    assert lib.hinm_calib_tile_part(C.byref(sh), 512, None, fake, 512, 1, None) == 1
    assert lib.hinm_calib_tile_part(C.byref(sh), 512, fake, fake, 100, 1, None) == 2      # ldx below N
    assert lib.hinm_calib_tile_part(C.byref(sh), 512, fake, fake, 512, 3, None) == 5      # no such part
    sh16 = binding._shape(256, 512, 16, 256, "bf16")
    assert lib.hinm_calib_tile_part(C.byref(sh16), 512, fake, fake, 512, 1, None) != 0    # no prepared form at V = 16
    assert lib.hinm_calib_tile_part(C.byref(sh), 8, fake, fake, 8, 1, None) == 5          # few columns: another kernel


def test_apply_row_order_validation():
    lib = hinm.load_library()
    fake = 0x1000
    assert lib.hinm_apply_row_order(None, fake + 4096, fake, 4, 64, None) == 1
    assert lib.hinm_apply_row_order(fake, fake + 4096, None, 4, 64, None) == 1
    assert lib.hinm_apply_row_order(fake, fake, fake + 8192, 4, 64, None) == 2           # in place
    assert lib.hinm_apply_row_order(fake, fake + 4096, fake + 8192, 4, 66, None) == 2    # row bytes not a multiple of 4
    assert lib.hinm_apply_row_order(fake, fake + 4096, fake + 8192, 0, 64, None) == 2


def test_tile_order_validation():
    lib = hinm.load_library()
    fake = 0x1000
    sh = binding._shape(64, 96, 16, 48, "f16")
    assert lib.hinm_tile_order(C.byref(sh), None, fake, None) == 1
    assert lib.hinm_tile_order(C.byref(sh), fake, None, None) == 1
    assert lib.hinm_tile_order(C.byref(sh), fake + 2, fake, None) == 2
    assert lib.hinm_tile_order(C.byref(binding._shape(64, 96, 16, 50, "f16")), fake, fake, None) == 2   # Kv % 8
    big = binding._shape(16, 400000, 16, 48, "f16")
    assert lib.hinm_tile_order(C.byref(big), fake, fake, None) == 5


def test_chain_validation():
    lib = hinm.load_library()
    fake = 0x1000
    mk = lambda M, K, dtype=0, flags=0: binding._Layer(binding._Shape(M, K, 16, K // 2, dtype), fake, fake, fake,
                                                       None, None, flags)
    out = C.c_size_t(0)
    two = (binding._Layer * 2)(mk(256, 128), mk(64, 256))
    assert lib.hinm_chain_sizes(2, two, 100, C.byref(out)) == 0
    assert out.value == 256 * 104 * 2           # one intermediate, columns padded to 8
    three = (binding._Layer * 3)(mk(256, 128), mk(64, 256), mk(32, 64))
    assert lib.hinm_chain_sizes(3, three, 8, C.byref(out)) == 0
    assert out.value == 2 * 256 * 8 * 2
    bad = (binding._Layer * 2)(mk(256, 128), mk(64, 128))          # K of layer 2 != M of layer 1
    assert lib.hinm_chain_sizes(2, bad, 8, C.byref(out)) == 2
    bad = (binding._Layer * 2)(mk(256, 128), mk(64, 256, dtype=1))  # mixed dtypes
    assert lib.hinm_chain_sizes(2, bad, 8, C.byref(out)) == 3
    bad = (binding._Layer * 2)(mk(256, 128, flags=2), mk(64, 256))  # fp32 output before the last layer
    assert lib.hinm_chain_sizes(2, bad, 8, C.byref(out)) == 5
    assert lib.hinm_chain(2, two, 8, fake, 8, fake, 8, None, 0, None) == 4   # scratch missing


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libhinm.so"))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.hinm_pack_sizes(256, 256, 16, 128, "f16")
