"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments and call orders, lays tiles out as documented, and
counts products as the closed forms say."""
import os
import re

import numpy as np
import pytest

import workloads as W
from paper_2508_14848_amd import gemm_mp as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gemm_mp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(gemm_mp_[a-z_]+)\s*\(", header)))
    assert declared == sorted(G.EXPORTS)
    L = G.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_create_rejects_bad_sizes():
    for args in ((0, 256, 256, 128), (256, 256, 256, 0), (256, 0, 300, 128), (256, 256, 256, 64),
                 (256, 256, 256, 96), (-256, 256, 256, 128), (1 << 15, 1 << 15, 1 << 15, 16384),
                 (128 * 32768, 128, 128, 128)):
        with pytest.raises(G.GemmMPError) as e:
            G.GemmMP(*args)
        assert e.value.status == G.EINVAL
    G.GemmMP(256, 512, 384, 128).destroy()
    # sizes off the tile grid: tile counts round up, maps have that shape
    g = G.GemmMP(300, 520, 777, 128)
    assert g.tiles("A") == (3, 7) and g.tiles("B") == (7, 5) and g.tiles("C") == (3, 5)
    g.set_precision_map("A", np.zeros((3, 7), dtype=np.uint16))
    assert g.storage_bytes("A") == 3 * 7 * 128 * 128 * 8          # whole tiles are stored
    with pytest.raises(G.GemmMPError) as e:
        g.set_precision_map("B", np.zeros((6, 5), dtype=np.uint16))
    assert e.value.status == G.EINVAL
    g.destroy()
    g = G.GemmMP(1, 1, 1, 128)
    assert g.tiles("C") == (1, 1)
    g.set_transposed("A", 1)
    g.set_transposed("B", 0)
    with pytest.raises(G.GemmMPError) as e:
        g.set_transposed("C", 1)                       # C is always given as it is
    assert e.value.status == G.EINVAL
    g.destroy()


def test_map_validation_and_call_order():
    g = G.GemmMP(512, 256, 384, 128)
    with pytest.raises(G.GemmMPError) as e:
        g.storage_bytes("A")
    assert e.value.status == G.ESTATE
    with pytest.raises(G.GemmMPError) as e:
        g.get_stats()
    assert e.value.status == G.ESTATE
    with pytest.raises(G.GemmMPError) as e:
        g.set_precision_map("A", np.zeros((3, 4), np.uint16))          # A is 4 x 3 tiles
    assert e.value.status == G.EINVAL
    with pytest.raises(G.GemmMPError) as e:
        g.set_precision_map("A", np.full((4, 3), 8, np.uint16))        # code out of range
    assert e.value.status == G.EINVAL
    with pytest.raises(G.GemmMPError) as e:
        g.set_precision_map("X", np.zeros((4, 3), np.uint16))
    assert e.value.status == G.EINVAL
    with pytest.raises(G.GemmMPError) as e:
        g.set_policy(7)
    assert e.value.status == G.EINVAL
    g.set_precision_map("A", np.zeros((4, 3), np.uint16))
    with pytest.raises(G.GemmMPError) as e:
        g.bind_storage("A", 0, 1 << 20)                                 # null buffer
    assert e.value.status == G.EINVAL
    with pytest.raises(G.GemmMPError) as e:
        g.bind_storage("A", 4096 + 8, 1 << 30)                          # misaligned
    assert e.value.status == G.EINVAL
    with pytest.raises(G.GemmMPError) as e:
        g.bind_storage("A", 4096, 100)                                  # too small
    assert e.value.status == G.EINVAL
    with pytest.raises(G.GemmMPError) as e:
        g.run(1.0, 0.0)
    assert e.value.status == G.ESTATE
    with pytest.raises(G.GemmMPError) as e:
        g.pack_tiles("B", 4096, 256)
    assert e.value.status == G.ESTATE
    assert "order" in G.strerror(G.ESTATE) and G.strerror(0) == "success"


def test_packed_layout_offsets_and_sizes():
    g = G.GemmMP(256, 384, 512, 128)
    pmap = np.array([[0, 1, 2, 3], [3, 2, 1, 0]], dtype=np.uint16)
    g.set_precision_map("A", pmap)
    sizes = [128 * 128 * (8 >> int(p)) for p in pmap.ravel()]
    off = 0
    for t, (I, J) in enumerate((i, j) for i in range(2) for j in range(4)):
        o, prec, _ = g.tile_info("A", I, J, want_exp=False)
        assert o == off and o % 256 == 0 and prec == pmap[I, J]
        off += sizes[t]
    assert g.storage_bytes("A") == off
    with pytest.raises(G.GemmMPError) as e:
        g.tile_info("A", 2, 0, want_exp=False)
    assert e.value.status == G.EINVAL
    with pytest.raises(G.GemmMPError) as e:
        g.tile_info("A", 0, 2, want_exp=True)        # FP16 tile, exponent unknown before packing
    assert e.value.status == G.ESTATE
    assert g.tile_info("A", 0, 0, want_exp=True)[2] == 0


def test_c_tiles_in_fp16_or_fp8_carry_an_fp32_staging_copy_behind_the_packed_tiles():
    nb = 256
    g = G.GemmMP(2 * nb, 3 * nb, nb, nb)
    mC = np.array([[G.FP64, G.FP16, G.FP32], [G.FP8_E4M3, G.FP32, G.FP16]], dtype=np.uint16)
    g.set_precision_map("C", mC)
    packed = sum(nb * nb * (8 >> int(p)) for p in mC.ravel())
    assert g.storage_bytes("C") == packed + 3 * nb * nb * 4
    off = 0
    for I in range(2):
        for J in range(3):
            o, prec, _ = g.tile_info("C", I, J, want_exp=False)
            assert o == off and prec == mC[I, J]                   # the packed tiles lie as for A
            off += nb * nb * (8 >> int(mC[I, J]))
    # the same codes on A need no staging
    g.set_precision_map("A", mC[:, :1])
    assert g.storage_bytes("A") == sum(nb * nb * (8 >> int(p)) for p in mC[:, 0])
    # products of such tiles are counted as an FP32 tile's, under both policies
    g.set_precision_map("A", np.full((2, 1), G.FP64, dtype=np.uint16))
    g.set_precision_map("B", np.full((1, 3), G.FP16, dtype=np.uint16))
    assert g.get_stats()["products"] == [1, 5, 0, 0]
    g.set_policy(G.POLICY_C_TILE)
    assert g.get_stats()["products"] == [1, 5, 0, 0]
    assert g.get_stats()["tiles"][2] == [1, 2, 2, 1]
    g.destroy()


def test_bf16_codes_layout_products_and_conversion_plan():
    """BF16 (code 4): two bytes per element, no staging on A or B; the product precision equals
    the oracle's for every triple and both policies; BF16 products are counted apart; the
    sender-side plan holds an FP32 copy of a BF16 tile that meets an FP32 tile and a BF16 copy
    of an FP8 tile that meets a BF16 tile."""
    from oracle import gemm_mp_oracle as orc
    for pA in range(5):
        for pB in range(5):
            for pC in range(7):
                for policy in (G.POLICY_OPERAND, G.POLICY_C_TILE):
                    assert G.product_precision(pA, pB, pC, policy) == orc.product_precision(pA, pB, pC, policy)
    nb = 128
    g = G.GemmMP(2 * nb, 2 * nb, 2 * nb, nb)
    full = lambda p: np.full((2, 2), p, dtype=np.uint16)
    g.set_precision_map("A", full(G.BF16))
    assert g.storage_bytes("A") == 4 * nb * nb * 2
    g.set_precision_map("B", full(G.BF16))
    g.set_precision_map("C", full(G.FP32))
    st = g.get_stats()
    assert st["products"] == [0, 0, 0, 0] and st["products_bf16"] == 8 and st["flops_bf16"] == 8 * 2.0 * nb ** 3
    assert st["tiles_bf16"] == [4, 4, 0] and g.conversion_bytes() == 0
    g.set_precision_map("B", full(G.FP32))                    # FP32 products: A's tiles need FP32 copies
    assert g.get_stats()["products"] == [0, 8, 0, 0] and g.conversion_bytes() == 4 * nb * nb * 4
    g.set_precision_map("B", full(G.FP16))                    # FP16 with BF16: FP32 products, copies of both
    assert g.get_stats()["products"] == [0, 8, 0, 0] and g.conversion_bytes() == 8 * nb * nb * 4
    g.set_precision_map("B", full(G.FP8_E4M3))                # BF16 products: B's tiles need BF16 copies
    assert g.get_stats()["products_bf16"] == 8 and g.conversion_bytes() == 4 * nb * nb * 2
    g.set_precision_map("C", full(G.BF16))                    # a BF16 C tile: stored BF16 behind FP32 staging
    assert g.storage_bytes("C") == 4 * nb * nb * (2 + 4) and g.get_stats()["products_bf16"] == 8
    g.destroy()


def test_mxfp8_codes_layout_and_where_this_build_runs_them():
    """MXFP8 (code 5): nb^2 element bytes plus nb^2/32 scale bytes per tile (a C tile gets an FP32 staging copy besides); the
    product precision equals the oracle's; tiles made of MXFP8 x MXFP8 products only are cut into
    256 x 256 regions; statistics count such products apart."""
    from oracle import gemm_mp_oracle as orc
    for pA in range(7):
        for pB in range(7):
            for pC in range(7):
                for policy in (G.POLICY_OPERAND, G.POLICY_C_TILE):
                    assert G.product_precision(pA, pB, pC, policy) == orc.product_precision(pA, pB, pC, policy)
    nb = 512
    g = G.GemmMP(2 * nb, 2 * nb, 3 * nb, nb)
    g.set_precision_map("A", np.full((2, 3), G.MXFP8, dtype=np.uint16))
    assert g.storage_bytes("A") == 6 * (nb * nb + nb * nb // 32)
    o, prec, _ = g.tile_info("A", 0, 1, want_exp=False)
    assert o == nb * nb + nb * nb // 32 and prec == G.MXFP8
    # a block-scaled C tile: its packed form, and an FP32 staging copy behind all packed tiles
    g.set_precision_map("C", np.array([[G.MXFP8, G.FP32], [G.MXFP4, G.FP64]], dtype=np.uint16))
    packed = (nb * nb + nb * nb // 32) + 4 * nb * nb + (nb * nb // 2 + nb * nb // 32) + 8 * nb * nb
    assert g.storage_bytes("C") == packed + 2 * 4 * nb * nb
    g.set_precision_map("B", np.full((3, 2), G.MXFP8, dtype=np.uint16))
    g.set_precision_map("C", np.full((2, 2), G.FP32, dtype=np.uint16))
    st = g.get_stats()
    assert st["products_mxfp8"] == 12 and st["products"] == [0, 0, 0, 0] and st["tiles_mxfp8"] == [6, 6, 0]
    assert st["flops_mxfp8"] == 12 * 2.0 * nb ** 3 and st["work_items"] == 4 * (nb // 256) ** 2
    assert g.conversion_bytes() == 0
    # MXFP4 (code 6): half a byte per element; block-scaled kernel at tile sizes that are multiples of 512
    g.set_precision_map("A", np.full((2, 3), G.MXFP4, dtype=np.uint16))
    g.set_precision_map("B", np.full((3, 2), G.MXFP4, dtype=np.uint16))
    assert g.storage_bytes("A") == 6 * (nb * nb // 2 + nb * nb // 32)
    st = g.get_stats()
    assert st["products_mxfp4"] == 12 and st["tiles_mxfp4"] == [6, 6, 0] and st["work_items"] == 4 * (nb // 256) ** 2
    assert g.conversion_bytes() == 0
    # MXFP6 (code 7): three quarters of a byte per element; block-scaled kernel at multiples of 256
    g.set_precision_map("A", np.full((2, 3), G.MXFP6, dtype=np.uint16))
    g.set_precision_map("B", np.full((3, 2), G.MXFP6, dtype=np.uint16))
    assert g.storage_bytes("A") == 6 * (nb * nb * 3 // 4 + nb * nb // 32)
    o, prec, _ = g.tile_info("A", 1, 0, want_exp=False)
    assert o == 3 * (nb * nb * 3 // 4 + nb * nb // 32) and prec == G.MXFP6
    st = g.get_stats()
    assert st["products_mxfp6"] == 12 and st["tiles_mxfp6"] == [6, 6, 0] and st["work_items"] == 4 * (nb // 256) ** 2
    assert st["launch_items"] == [0, 0, 0, 0, 0, 0, 0, st["work_items"]] and st["flops_mxfp6"] == 12 * 2.0 * nb ** 3
    assert g.conversion_bytes() == 0
    g.set_precision_map("A", np.full((2, 3), G.MXFP4, dtype=np.uint16))
    g.set_precision_map("B", np.full((3, 2), G.MXFP4, dtype=np.uint16))
    g.set_precision_map("B", np.full((3, 2), G.MXFP8, dtype=np.uint16))      # MXFP4 with MXFP8: FP32 on copies of both
    assert g.get_stats()["products"] == [0, 12, 0, 0] and g.conversion_bytes() == 12 * nb * nb * 4
    g.destroy()
    g = G.GemmMP(256, 256, 256, 256)                                          # 256 is no multiple of 512: copies
    for k in "AB":
        g.set_precision_map(k, np.full((1, 1), G.MXFP4, dtype=np.uint16))
    g.set_precision_map("C", np.full((1, 1), G.FP32, dtype=np.uint16))
    assert g.get_stats()["products_mxfp4"] == 1 and g.conversion_bytes() == 2 * 256 * 256 * 4
    g.destroy()


def test_product_precision_and_stats_closed_forms():
    for pA in range(4):
        for pB in range(4):
            for pC in range(2):
                assert G.product_precision(pA, pB, pC, G.POLICY_C_TILE) == pC
                assert G.product_precision(pA, pB, pC, G.POLICY_OPERAND) == max(pC and 1, min(pA, pB))
    assert G.product_precision(7, 0, 0) == -1 and G.product_precision(0, 0, 7) == -1
    w = W.tiny()
    g = G.GemmMP(w.M, w.N, w.K, w.nb)
    for k, m in (("A", w.mapA), ("B", w.mapB), ("C", w.mapC)):
        g.set_precision_map(k, m)
    st = g.get_stats()
    assert st["products"] == [28, 26, 10, 0] and st["work_items"] == 16 * 4
    assert st["flops"][0] == 28 * 2.0 * 256 ** 3
    assert st["tiles"][0] == [4, 6, 6, 0] and st["tiles"][2] == [16, 0, 0, 0]
    assert st["packed_bytes"][2] == 1024 * 1024 * 8
    g.set_policy(G.POLICY_C_TILE)
    assert g.get_stats()["products"] == [64, 0, 0, 0]
    w = W.random_maps()
    g = G.GemmMP(w.M, w.N, w.K, w.nb)
    for k, m in (("A", w.mapA), ("B", w.mapB), ("C", w.mapC)):
        g.set_precision_map(k, m)
    st = g.get_stats()
    assert sum(st["products"]) == 16 ** 3 and st["work_items"] == 256 * 16
    n64 = int((w.mapC == 0).sum())
    g.set_policy(G.POLICY_C_TILE)
    assert g.get_stats()["products"] == [n64 * 16, (256 - n64) * 16, 0, 0]


def test_fp8_only_tiles_are_scheduled_in_large_regions():
    """An FP32 C tile whose every product multiplies two FP8 tiles at FP8 is cut into 256 x 256
    regions, every other tile into 128 x 128 ones; a tile size that is not a multiple of 256
    keeps the small regions everywhere."""
    FP64, FP32, FP16, FP8 = 0, 1, 2, 3
    for nb, want_big in ((512, True), (384, False)):
        MT, NT, KT = 3, 2, 2
        g = G.GemmMP(MT * nb, NT * nb, KT * nb, nb)
        mA = np.full((MT, KT), FP8, dtype=np.uint16)
        mB = np.full((KT, NT), FP8, dtype=np.uint16)
        mC = np.full((MT, NT), FP32, dtype=np.uint16)
        mA[2, 1] = FP16                       # tile row 2: a converting product, small regions
        mC[0, 1] = FP64                       # an FP64 tile: small regions
        for k, m in (("A", mA), ("B", mB), ("C", mC)):
            g.set_precision_map(k, m)
        big = 3 if want_big else 0            # tiles (0,0), (1,0), (1,1)
        small = MT * NT - big
        assert g.get_stats()["work_items"] == small * (nb // 128) ** 2 + big * (nb // 256) ** 2
        g.set_policy(G.POLICY_C_TILE)         # every product at FP32 / FP64: no FP8 product left
        assert g.get_stats()["work_items"] == MT * NT * (nb // 128) ** 2


def test_sender_side_conversion_plan_closed_forms():
    """Workspace size = one copy per (tile, product precision != stored precision) that some task
    needs; host logic only."""
    nb = 128
    g = G.GemmMP(2 * nb, 2 * nb, 2 * nb, nb)
    with pytest.raises(G.GemmMPError) as e:
        g.conversion_bytes()
    assert e.value.status == G.ESTATE
    full = lambda p: np.full((2, 2), p, dtype=np.uint16)
    g.set_precision_map("A", full(G.FP64))
    g.set_precision_map("B", full(G.FP32))
    g.set_precision_map("C", full(G.FP64))
    # every product is FP64: the four FP32 tiles of B need an FP64 copy, A needs nothing
    assert g.conversion_bytes() == 4 * nb * nb * 8
    g.set_precision_map("C", full(G.FP32))
    # now every product is FP32: the four FP64 tiles of A need an FP32 copy
    assert g.conversion_bytes() == 4 * nb * nb * 4
    mC = np.array([[G.FP64, G.FP32], [G.FP32, G.FP32]], dtype=np.uint16)
    g.set_precision_map("C", mC)
    # C(0,0) runs FP64 products: B(0,0), B(1,0) up; all other C tiles run FP32: A(0,:) and A(1,:) down
    assert g.conversion_bytes() == 2 * nb * nb * 8 + 4 * nb * nb * 4
    g.set_precision_map("A", full(G.FP8_E4M3))
    g.set_precision_map("B", full(G.FP16))
    g.set_precision_map("C", full(G.FP32))
    # FP16 products: the FP8 tiles of A get FP16 copies
    assert g.conversion_bytes() == 4 * nb * nb * 2
    g.set_precision_map("B", full(G.FP8_E4M3))
    assert g.conversion_bytes() == 0
    assert g.get_stats()["converted_tiles"] == 0
    with pytest.raises(G.GemmMPError) as e:
        g.convert_tiles(0, 0, None)               # nothing is packed yet
    assert e.value.status == G.ESTATE
    g.clear_conversion()


def test_isa_check_flags_a_copy_of_an_accumulator_inside_a_run_of_assembly_matrix_instructions(tmp_path):
    """The build's machine-code check on three made-up basic blocks: a clean run, a run with a
    register copy of one of its accumulators in the middle, and a copy behind the run."""
    from paper_2508_14848_amd import check_isa
    clean = "\n".join(["v_mfma_f32_16x16x4_f32 v[192:195], v1, v2, v[192:195]", "ds_read_b128 v[10:13], v5",
                       "v_mfma_f32_16x16x4_f32 a[4:7], v1, v3, a[4:7]", "s_nop 11", "v_accvgpr_read_b32 v9, a4"])
    dirty = "\n".join(["v_mfma_f32_16x16x4_f32 a[4:7], v1, v2, a[4:7]", "v_accvgpr_mov_b32 a9, a5",
                       "v_mfma_f32_16x16x4_f32 a[4:7], v1, v3, a[4:7]"])
    other = "\n".join(["v_mfma_f64_16x16x4_f64 a[0:7], v[0:1], v[2:3], a[0:7]", "v_accvgpr_mov_b32 a9, a5"])
    p = tmp_path / "k.s"
    p.write_text(".LBB0_1:\n" + clean + "\ns_cbranch_scc1 .LBB0_1\n.LBB0_2:\n" + other + "\n")
    assert check_isa.violations(str(p)) == (1, [])
    p.write_text(".LBB0_1:\n" + clean + "\ns_branch .LBB0_3\n.LBB0_2:\n" + dirty + "\ns_endpgm\n")
    n, bad = check_isa.violations(str(p))
    assert n == 2 and bad == ["v_accvgpr_mov_b32 a9, a5"]
