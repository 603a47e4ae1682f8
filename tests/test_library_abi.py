"""The C-ABI library loads, exports what include/slim.h declares, and its
host-side logic (size queries, argument validation) behaves as documented.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2410_09615_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "slim.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slim_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings():
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert B.slim_status_string(code)
    assert B.slim_status_string(-99) == "unknown status"


def test_rank_pad_and_sizes():
    assert [B.slim_rank_pad(r) for r in (0, 1, 32, 33, 51, 410, 512, 820)] == [0, 32, 32, 64, 64, 416, 512, 832]
    s = B.slim_packed_sizes(4096, 4096, 410)
    assert s == {"qvals": 4096 * 1024, "meta": 4096 * 512, "scale": 4096 * 4, "rank_pad": 416,
                 "L": 4096 * 416 * 2, "R": 416 * 4096 * 2}
    for bad in ((0, 512, 1), (8, 4, 0), (8, 12, 0), (8, 16, -1)):
        with pytest.raises(B.SlimError) as e:
            B.slim_packed_sizes(*bad)
        assert e.value.status == B.SLIM_ERR_SHAPE


def test_workspace_query():
    layer = B.slim_layer(B.slim_shape(4096, 4096, 410), None, None, None, None, None, 416, 16, None, None, None, None)
    out = ctypes.c_size_t()
    assert B.lib().slim_workspace_bytes(ctypes.byref(layer), 16, out) == 0
    # at least T (fp32 [16][416]) and the quantized-term buffer (fp32 [16][4096])
    assert out.value >= 16 * 416 * 4 + 16 * 4096 * 4
    big = ctypes.c_size_t()
    assert B.lib().slim_workspace_bytes(ctypes.byref(layer), 2048, big) == 0
    assert big.value >= 2048 * 416 * 2
    # 4-bit adapters: prefill reads the codes itself and needs no room for an fp16 copy of them; a decode call
    # may fall back on the two-launch kernels, which read fp16: room for both adapters then
    q4 = B.slim_layer(B.slim_shape(4096, 4096, 410), None, None, None, None, None, 416, 4, None, None, None, None)
    q4_big, q4_dec = ctypes.c_size_t(), ctypes.c_size_t()
    assert B.lib().slim_workspace_bytes(ctypes.byref(q4), 2048, q4_big) == 0 and q4_big.value == big.value
    assert B.lib().slim_workspace_bytes(ctypes.byref(q4), 16, q4_dec) == 0
    assert q4_dec.value >= out.value + 2 * 4096 * 416 * 2
    layer.rank_pad = 410                                # not slim_rank_pad(rank)
    assert B.lib().slim_workspace_bytes(ctypes.byref(layer), 16, out) == B.SLIM_ERR_SHAPE
    assert B.lib().slim_workspace_bytes(None, 16, out) == B.SLIM_ERR_NULL


def test_argument_validation_returns_codes_before_any_launch():
    lib = B.lib()
    shape = B.slim_shape(128, 256, 0)
    a = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    assert lib.slim_pack(None, shape, a, a, a, None) == B.SLIM_ERR_NULL
    assert lib.slim_pack(a, B.slim_shape(128, 12, 0), a, a, a, None) == B.SLIM_ERR_SHAPE
    assert lib.slim_pack(ctypes.c_void_p(0x1004), shape, a, a, a, None) == B.SLIM_ERR_ALIGN
    assert lib.slim_unpack(a, None, shape, a, a, None) == B.SLIM_ERR_NULL
    assert lib.slim_pack_adapters(a, a, shape, a, a, None) == B.SLIM_ERR_SHAPE      # rank 0
    layer = B.slim_layer(shape, 0x1000, 0x1000, 0x1000, None, None, 0)
    for fn in (lib.slim_linear_gemv, lib.slim_linear_gemm):
        assert fn(None, a, 1, a, a, 1 << 20, None) == B.SLIM_ERR_NULL
        assert fn(ctypes.byref(layer), a, 0, a, a, 1 << 20, None) == B.SLIM_ERR_SHAPE
        assert fn(ctypes.byref(layer), a, 1, a, a, 16, None) == B.SLIM_ERR_WORKSPACE
        assert fn(ctypes.byref(layer), a, 1, a, None, 0, None) == B.SLIM_ERR_WORKSPACE
    assert lib.slim_linear_gemv(ctypes.byref(layer), a, 17, a, a, 1 << 20, None) == B.SLIM_ERR_SHAPE
    odd = B.slim_layer(B.slim_shape(128, 192, 0), 0x1000, 0x1000, 0x1000, None, None, 0)
    assert lib.slim_linear_gemv(ctypes.byref(odd), a, 1, a, a, 1 << 20, None) == B.SLIM_ERR_SHAPE   # k % 128
    withrank = B.slim_layer(B.slim_shape(128, 256, 8), 0x1000, 0x1000, 0x1000, None, None, 32)
    assert lib.slim_linear_gemm(ctypes.byref(withrank), a, 4, a, a, 1 << 20, None) == B.SLIM_ERR_NULL
    assert lib.slim_lowrank(a, 4, a, a, B.slim_shape(128, 256, 0), 0, a, 0, a, 1 << 20, None) == B.SLIM_ERR_SHAPE
    assert lib.slim_lowrank(a, 4, a, a, B.slim_shape(128, 256, 8), 8, a, 0, a, 1 << 20, None) == B.SLIM_ERR_SHAPE
    # the 8-bit-input forms
    gf = lib.slim_linear_gemm_fp8
    assert gf(None, a, a, 0, 4, a, a, 1 << 20, None) == B.SLIM_ERR_NULL
    assert gf(ctypes.byref(layer), a, None, 0, 4, a, a, 1 << 20, None) == B.SLIM_ERR_NULL          # no scale
    assert gf(ctypes.byref(layer), a, a, 2, 4, a, a, 1 << 20, None) == B.SLIM_ERR_SHAPE            # format is 0 or 1
    assert gf(ctypes.byref(layer), a, a, 0, 0, a, a, 1 << 20, None) == B.SLIM_ERR_SHAPE
    assert gf(ctypes.byref(layer), ctypes.c_void_p(0x1004), a, 0, 4, a, a, 1 << 20, None) == B.SLIM_ERR_ALIGN
    assert gf(ctypes.byref(layer), a, a, 1, 4, a, a, 16, None) == B.SLIM_ERR_WORKSPACE
    qc = lib.slim_input_quant_fp8_codes
    assert qc(a, 16, None, None, a, a, 1024, None) == B.SLIM_ERR_NULL                              # nothing to write
    assert qc(a, 0, a, a, a, a, 1024, None) == B.SLIM_ERR_SHAPE
    assert qc(a, 16, a, ctypes.c_void_p(0x1001), a, a, 1024, None) == B.SLIM_ERR_ALIGN
    assert qc(a, 16, None, a, a, a, 8, None) == B.SLIM_ERR_WORKSPACE
    assert lib.slim_input_quant_fp8(a, 16, None, a, a, 1024, None) == B.SLIM_ERR_NULL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libslim.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_adapter_computation_workspace_query_and_validation():
    lib = B.lib()
    out = ctypes.c_size_t()
    assert lib.slim_adapters_workspace_bytes(B.slim_shape(4096, 4096, 410), out) == 0
    # the error saliency (fp32 [n][k]) and three blocks of rank_pad columns at least
    assert out.value >= 4 * 4096 * 4096 + 3 * 4 * 4096 * 416
    for bad in ((4096, 4096, 0), (64, 4096, 65), (4096, 4100, 16), (4096, 4096, 2000)):
        assert lib.slim_adapters_workspace_bytes(B.slim_shape(*bad), out) == B.SLIM_ERR_SHAPE
    assert lib.slim_adapters_workspace_bytes(B.slim_shape(4096, 4096, 410), None) == B.SLIM_ERR_NULL
    assert lib.slim_compute_adapters(None, None, None, None, B.slim_shape(128, 128, 8), None, 0, 1, None, None, None,
                                     None, 0, None) == B.SLIM_ERR_NULL


def test_probe_validation():
    lib = B.lib()
    fl = ctypes.c_double()
    assert lib.slim_probe_read(None, 1 << 20, 1, 0, None, None) == B.SLIM_ERR_NULL
    assert lib.slim_probe_mfma(0, 16, 16, None, fl, None) == B.SLIM_ERR_NULL


def test_input_quant_validation():
    lib = B.lib()
    assert lib.slim_input_quant_fp8(None, 16, None, None, None, 0, None) == B.SLIM_ERR_NULL


def test_decode_plan_of_the_configured_shapes(decode_override):
    """Host logic of slim_linear_gemv: every configured layer takes the one-launch path at every token
    count, within what a compute unit holds (1024 threads, 160 KiB of LDS, 16 wavefronts), with all
    workgroups resident at once and every row tile covered."""
    from paper_2410_09615_amd import workloads as wl
    decode_override("auto", 0)
    for shp in (wl.TINY, wl.L7B_ATTN, wl.L7B_UP, wl.L7B_DOWN, wl.L13B_ATTN, wl.L13B_UP, wl.L70B_ATTN, wl.L70B_UP):
        for m in (1, 2, 4, 8, 16):
            p = B.slim_decode_plan(shp.n, shp.k, shp.r, m)
            assert p["path"] == 2, (shp.name, m)
            assert p["threads"] % 64 == 0 and p["threads"] <= 1024
            assert p["threads"] == 64 * (p["working_wavefronts"] + p["helper_wavefronts"])
            assert p["lds_bytes"] <= 160 * 1024
            per_cu = min(16 // (p["threads"] // 64), (160 * 1024) // p["lds_bytes"])
            assert p["workgroups"] == p["r_workgroups"] + p["y_workgroups"] <= 256 * per_cu
            assert p["r_workgroups"] == (B.slim_rank_pad(shp.r) // 16) * p["r_shares"] <= 512
            tiles = (shp.n + 15) // 16
            assert p["y_workgroups"] * (p["working_wavefronts"] // p["wavefronts_per_row_tile"]) >= tiles
            assert p["chunk_inputs"] * p["chunks"] >= shp.k and p["chunk_inputs"] % 1024 == 0
            if p["chunks"] > 1:
                assert B.slim_rank_pad(shp.r) <= p["chunk_inputs"]        # T takes the place of an X buffer
    # forced paths and errors
    decode_override("parts")
    assert B.slim_decode_plan(4096, 4096, 410, 1)["path"] == 0
    decode_override("roles")
    assert B.slim_decode_plan(4096, 4096, 410, 1)["path"] == 1
    decode_override("auto")
    for bad in ((4, 0), (-2, 0), (0, 8), (0, 161)):
        assert B.lib().slim_decode_override(*bad) == B.SLIM_ERR_SHAPE
    with pytest.raises(B.SlimError):
        B.slim_decode_plan(4096, 4096, 410, 17)
    with pytest.raises(B.SlimError):
        B.slim_decode_plan(4096, 4100, 410, 1)
    # a reduced LDS budget (what the chunk tests use) forces chunks
    for n, k, r, m, lds_kb in [(1000, 4096, 100, 16, 96), (1000, 4096, 100, 16, 72), (520, 11008, 410, 8, 64),
                               (300, 2176, 37, 5, 24), (2049, 8192, 33, 16, 160), (64, 3072, 0, 16, 70)]:
        decode_override("auto", lds_kb)
        p = B.slim_decode_plan(n, k, r, m)
        assert p["path"] == 2 and p["chunks"] > 1 and p["lds_bytes"] <= lds_kb * 1024, (n, k, r, m, lds_kb)


def test_static_scratch_call_validates_on_the_host():
    """slim_linear_gemv_static checks arguments and the size of its own scratch array before anything
    touches a device."""
    lib = B.lib()
    a = ctypes.c_void_p(0x1000)
    layer = B.slim_layer(B.slim_shape(128, 256, 0), 0x1000, 0x1000, 0x1000, None, None, 0)
    assert lib.slim_linear_gemv_static(None, a, 1, a, None) == B.SLIM_ERR_NULL
    assert lib.slim_linear_gemv_static(ctypes.byref(layer), a, 0, a, None) == B.SLIM_ERR_SHAPE
    assert lib.slim_linear_gemv_static(ctypes.byref(layer), a, 17, a, None) == B.SLIM_ERR_SHAPE
    assert lib.slim_linear_gemv_static(ctypes.byref(layer), ctypes.c_void_p(0x1004), 1, a, None) == B.SLIM_ERR_ALIGN
    # a layer whose decode call needs partial sums beyond the array: 16 tokens x 600000 rows of floats per slot
    huge = B.slim_layer(B.slim_shape(600000, 8192, 0), 0x1000, 0x1000, 0x1000, None, None, 0)
    out = ctypes.c_size_t()
    assert lib.slim_workspace_bytes(ctypes.byref(huge), 16, out) == 0 and out.value > (8 << 20)
    assert B.slim_decode_plan(600000, 8192, 0, 16)["path"] == 0
    assert lib.slim_linear_gemv_static(ctypes.byref(huge), a, 16, a, None) == B.SLIM_ERR_WORKSPACE


def test_decode_refuses_buffers_the_kernels_cannot_address():
    """The decode kernels use 32-bit byte offsets with 2^31 as "past the end": a layer with a buffer of 2 GiB
    or more is refused on the host (slim_linear_gemv and slim_lowrank alike), one just below is planned."""
    lib = B.lib()
    a = ctypes.c_void_p(0x1000)
    big = B.slim_layer(B.slim_shape(1 << 20, 8192, 0), 0x1000, 0x1000, 0x1000, None, None, 0)      # 2 GiB of codes
    assert lib.slim_linear_gemv(ctypes.byref(big), a, 1, a, a, 1 << 40, None) == B.SLIM_ERR_SHAPE
    wide = B.slim_shape(1 << 20, 1024, 1024)                                                       # L: 2 GiB
    assert lib.slim_lowrank(a, 4, a, a, wide, 1024, a, 0, a, 1 << 40, None) == B.SLIM_ERR_SHAPE
    assert B.slim_decode_plan((1 << 20) - 32, 8192, 0, 1)["path"] in (0, 2)


def test_decode_plan_invariants_over_random_shapes():
    """Host logic only: for random layers and token counts the plan either declines (two-launch kernels) or
    describes a launch that fits a compute unit and covers every row tile and every input; the workspace
    and packed sizes are consistent with it."""
    import random
    rnd = random.Random(7)
    for _ in range(400):
        n = rnd.choice([rnd.randint(1, 300), rnd.randint(1, 40000)])
        k = 128 * rnd.randint(1, 120)
        r = rnd.choice([0, rnd.randint(1, min(n, k, 1100))])
        m = rnd.randint(1, 16)
        bits = rnd.choice([16, 4])
        p = B.slim_decode_plan(n, k, r, m, bits)
        rp = B.slim_rank_pad(r)
        layer = B.slim_layer(B.slim_shape(n, k, r), None, None, None, None, None, rp, bits, None, None, None, None)
        out = ctypes.c_size_t()
        assert B.lib().slim_workspace_bytes(ctypes.byref(layer), m, out) == 0
        assert out.value >= 256 + 3 * 16 * rp * 4 and out.value % 256 == 0
        sz = B.slim_packed_sizes(n, k, r)
        assert sz["qvals"] == 2 * sz["meta"] == ((n + 31) // 32) * ((k + 127) // 128) * 1024
        assert sz["rank_pad"] == rp and sz["L"] == ((n + 31) // 32 * 32) * rp * 2 and sz["R"] == rp * k * 2
        if p["path"] == 0:
            continue
        assert p["path"] == 2
        assert p["threads"] == 64 * (p["working_wavefronts"] + p["helper_wavefronts"]) <= 1024
        assert 0 < p["lds_bytes"] <= 160 * 1024
        per_cu = min(16 // (p["threads"] // 64), (160 * 1024) // p["lds_bytes"])
        assert per_cu >= 1 and p["workgroups"] == p["r_workgroups"] + p["y_workgroups"] <= 256 * per_cu
        assert p["r_workgroups"] == (rp // 16) * p["r_shares"] <= 512 and (p["r_shares"] in (1, 2, 4) or rp == 0)
        tpw = p["working_wavefronts"] // p["wavefronts_per_row_tile"]
        assert tpw >= 1 and p["working_wavefronts"] % p["wavefronts_per_row_tile"] == 0
        assert p["y_workgroups"] * tpw >= (n + 15) // 16
        assert p["chunk_inputs"] % 1024 == 0 and p["chunk_inputs"] * p["chunks"] >= k
        if p["chunks"] > 1:
            assert rp <= p["chunk_inputs"] and (p["chunk_inputs"] // 512) % p["wavefronts_per_row_tile"] == 0


def test_prefill_tile_order_covers_every_tile_once():
    """Host logic of slim_linear_gemm: the order in which workgroups take output tiles is a permutation of
    the tiles for every layer and token count (ragged edges included).  The 32 workgroups that share a
    die's L2 in a round (index mod 8) work on a block of 4 row tiles x 8 token tiles at the configured
    shapes, and over random shapes they touch no more distinct operand tiles than in index order (up to
    what a ragged last band costs)."""
    import random
    from paper_2410_09615_amd import workloads as wl

    def operand_tiles(n, m):
        tiles, n_full, order = B.slim_gemm_tile_order(n, m)
        tiles_o, tiles_t = (n + 511) // 512, (m + 127) // 128
        assert tiles == tiles_o * tiles_t and 0 <= n_full <= tiles, (n, m)
        assert sorted(order) == list(range(tiles)), (n, m)
        blocked, plain, worst = 0, 0, (0, 0)
        for start in range(0, n_full // 256 * 256, 256):
            for die in range(8):
                ws = range(start + die, start + 256, 8)
                rows, toks = {order[w] % tiles_o for w in ws}, {order[w] // tiles_o for w in ws}
                blocked += len(rows) + len(toks)
                plain += len({w % tiles_o for w in ws}) + len({w // tiles_o for w in ws})
                worst = max(worst, (len(rows), len(toks)))
        return blocked, plain, worst

    for shp, m in ((wl.L7B_UP, 2048), (wl.L7B_DOWN, 2048), (wl.L13B_ATTN, 4096), (wl.L13B_UP, 4096), (wl.L70B_ATTN, 4096),
                   (wl.L70B_UP, 4096)):
        blocked, plain, worst = operand_tiles(shp.n, m)
        assert worst[0] <= 8 and worst[1] <= 8 and blocked <= plain, (shp.name, worst, blocked, plain)
    rnd = random.Random(11)
    for n, m in [(1, 1), (513, 129), (512 * 9, 128 * 3), (40000, 300)] + [(rnd.randint(1, 40000), rnd.randint(1, 9000))
                                                                      for _ in range(80)]:
        blocked, plain, _ = operand_tiles(n, m)
        assert blocked <= 1.1 * plain + 8, (n, m, blocked, plain)
    for bad in ((0, 1), (1, 0)):
        out = (ctypes.c_int32 * 8)()
        assert B.lib().slim_gemm_tile_order(bad[0], bad[1], out, 8) == B.SLIM_ERR_SHAPE
    out = (ctypes.c_int32 * 3)()
    assert B.lib().slim_gemm_tile_order(1024, 256, out, 3) == B.SLIM_ERR_SHAPE
    assert B.lib().slim_gemm_tile_order(1024, 256, None, 100) == B.SLIM_ERR_NULL
