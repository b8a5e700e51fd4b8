"""Host-side checks of the C-ABI library: it loads without a GPU, exports every declared symbol,
and rejects bad arguments before touching the HIP runtime."""
import ctypes
import os
import re

import pytest

import paper_2107_06419_amd as fa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="flat_attn.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flat_attn_\w+)\s*\(", text)))


# every header under include/ and the library that implements it
HEADERS = {"flat_attn.h": fa.library_path, "flat_attn_probe.h": fa.probe_library_path}


def test_header_declares_the_expected_entry_points():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == sorted(HEADERS)
    names = declared_functions()
    for must in ("flat_attn_fwd", "flat_attn_fwd_f32", "flat_attn_unfused", "flat_attn_unfused_workspace_bytes",
                 "flat_attn_status_string", "flat_attn_version"):
        assert must in names
    assert not [n for n in names if "probe" in n], "the attention library carries no measurement aids"
    assert all("probe" in n for n in declared_functions("flat_attn_probe.h"))


def test_library_exports_every_declared_symbol():
    for header, path in HEADERS.items():
        if not os.path.exists(path()):
            pytest.fail(f"{path()} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(path())
        for name in declared_functions(header):
            assert hasattr(lib, name), f"{os.path.basename(path())} does not export {name}"


def test_binding_has_the_same_names():
    for header in HEADERS:
        for name in declared_functions(header):
            assert hasattr(fa, name), f"python binding lacks {name}"


def test_version_and_status_strings():
    assert fa.flat_attn_version() >= 100
    for code in range(0, -8, -1):
        s = fa.flat_attn_status_string(code)
        assert s and "unknown" not in s
    assert "unknown" in fa.flat_attn_status_string(-99)


def test_validation_happens_before_any_gpu_work():
    lib = fa.load_library()
    ok = (0x1000, 0x2000000, 0x4000000, 0x6000000)  # fake, aligned, far apart: never dereferenced on these paths

    def fwd(Q=ok[0], K=ok[1], V=ok[2], O=ok[3], B=1, H=1, N=8, d=64, scale=1.0, mask=0):
        return lib.flat_attn_fwd(Q, K, V, O, B, H, N, d, scale, mask, None)

    assert fwd(Q=None) == -1 and fwd(K=None) == -1 and fwd(V=None) == -1 and fwd(O=None) == -1
    assert fwd(B=0) == -2 and fwd(H=-1) == -2 and fwd(N=0) == -2
    assert fwd(d=48) == -3 and fwd(d=80) == -3 and fwd(d=512) == -3 and fwd(d=0) == -3 and fwd(mask=2) == -3 and fwd(mask=-1) == -3
    for d_ok in (32, 64, 96, 128, 256):   # every head dimension the fused bf16 kernel is built for gets past the d check
        assert fwd(d=d_ok, B=0) == -2
        assert fwd(d=d_ok, Q=ok[0] + 8) == -4
        assert lib.flat_attn_fwd_f32(ok[0] + 8, ok[1], ok[2], ok[3], 1, 1, 8, d_ok, 1.0, 0, None) == (-4 if d_ok in (64, 128) else -3)
    assert fwd(scale=-0.5) == -3 and fwd(scale=float("inf")) == -3 and fwd(scale=float("nan")) == -3
    assert fwd(Q=ok[0] + 8) == -4 and fwd(O=ok[3] + 2) == -4
    assert fwd(O=ok[0]) == -7 and fwd(O=ok[1] + 16) == -7
    assert fwd(B=1 << 20, H=1 << 20, N=1 << 20) == -2           # index overflow
    far = (0x1000, 1 << 40, 2 << 40, 3 << 40)
    assert fwd(*far, N=1 << 24, d=128) == -2 and fwd(*far, N=1 << 25, d=64) == -2  # one head reaches 4 GiB
    assert lib.flat_attn_fwd_f32(ok[0], ok[1], ok[2], ok[3], 1, 1, 8, 48, 1.0, 0, None) == -3

    assert fa.flat_attn_unfused_workspace_bytes(1, 16, 16384, 64) == 16 * 16384 * 16384 * 4
    assert fa.flat_attn_unfused_workspace_bytes(1, 8, 65536, 64) == 8 * 65536 * 65536 * 4
    assert fa.flat_attn_unfused_workspace_bytes(1, 1, 8, 96) == 0

    def unf(ws=0x8000000, ws_bytes=1 << 20, dtype=0, **kw):
        a = dict(Q=ok[0], K=ok[1], V=ok[2], O=ok[3], B=1, H=1, N=8, d=64, scale=1.0, mask=0)
        a.update(kw)
        return lib.flat_attn_unfused(a["Q"], a["K"], a["V"], a["O"], a["B"], a["H"], a["N"], a["d"], a["scale"], a["mask"],
                                     ws, ws_bytes, dtype, None)

    assert unf(ws=None) == -1
    assert unf(ws_bytes=8 * 8 * 4 - 1) == -5
    assert unf(dtype=1) == -3
    assert unf(ws=0x8000004) == -4
    assert unf(ws=ok[3]) == -7
    assert unf(N=0) == -2


def test_tile_shape_table_is_consistent():
    """The shape table is host data: index 0 is the default, every entry describes a launchable shape, and
    out-of-range queries are refused without touching a GPU."""
    lib = fa.load_library()
    assert fa.flat_attn_tile_shape_count(48) == 0 and fa.flat_attn_tile_shape_count(512) == 0
    for d in (32, 64, 96, 128, 256):
        n = fa.flat_attn_tile_shape_count(d)
        assert n >= (2 if d in (64, 128) else 1)
        seen = set()
        for idx in range(n):
            t = fa.flat_attn_tile_shape_get(d, idx).as_dict()
            assert t["d"] == d and t["keys_per_tile"] in ((32, 64, 128) if d == 64 else (32,) if d == 256 else (64,))
            if idx == 0:
                assert t["keys_per_tile"] == (32 if d == 256 else 64)
            assert t["rows_per_workgroup"] == t["wavefronts"] * t["rows_per_wavefront"]
            assert t["rows_per_wavefront"] in (32, 64) and 1 <= t["wavefronts"] <= 16
            assert t["lds_stages"] >= 3
            d_lds = 128 if d == 96 else d  # rows of 96 elements are padded to 128 in LDS
            assert t["lds_bytes"] == t["lds_stages"] * 2 * t["keys_per_tile"] * d_lds * 2 <= 160 * 1024  # K and V tiles, bf16
            assert 256 % t["rows_per_workgroup"] == 0 or t["rows_per_workgroup"] % 256 == 0
            key = (t["rows_per_workgroup"], t["wavefronts"], t["lds_stages"], t["keys_per_tile"])
            assert key not in seen
            seen.add(key)
        for bad in (-1, n):
            with pytest.raises(fa.FlatAttnError) as e:
                fa.flat_attn_tile_shape_get(d, bad)
            assert e.value.status == -2
            assert lib.flat_attn_fwd_tile(0x1000, 1 << 40, 2 << 40, 3 << 40, 1, 1, 8, d, 1.0, 0, bad, None) == -2
            assert lib.flat_attn_tile_shape_occupancy(d, bad) == -2
    assert lib.flat_attn_tile_shape_get(64, 0, None) == -1
    assert lib.flat_attn_tile_shape_occupancy(80, 0) == -3
    # the default shape is host arithmetic: large launches take index 0, small ones the 128-row shape
    assert fa.flat_attn_tile_shape_default(1, 16, 16384, 64, 0) == 0 and fa.flat_attn_tile_shape_default(2, 8, 8192, 128, 1) == 0
    assert fa.flat_attn_tile_shape_default(1, 12, 512, 64, 0) == 7 and fa.flat_attn_tile_shape_default(1, 12, 512, 128, 1) == 2
    assert fa.flat_attn_tile_shape_default(1, 12, 256, 64, 0) == 0 and fa.flat_attn_tile_shape_default(1, 129, 512, 64, 0) == 0
    for d in (32, 64, 96, 128, 256):
        for B, H, N, mask in ((1, 1, 1, 0), (3, 7, 300, 1), (1, 12, 512, 0), (64, 12, 512, 1), (1, 16, 16384, 0), (2147483, 1000, 77, 1)):
            idx = fa.flat_attn_tile_shape_default(B, H, N, d, mask)
            assert 0 <= idx < fa.flat_attn_tile_shape_count(d)
            if idx:
                assert fa.flat_attn_tile_shape_get(d, idx).as_dict()["rows_per_workgroup"] == 128
    assert lib.flat_attn_tile_shape_default(0, 1, 1, 64, 0) == -2 and lib.flat_attn_tile_shape_default(1, 1, 1, 80, 0) == -3
    assert lib.flat_attn_tile_shape_default(1, 1, 1, 64, 2) == -3 and lib.flat_attn_tile_shape_default(65536, 65536, 1, 64, 0) == -2
    d64, d128 = fa.flat_attn_tile_shape_get(64, 0).as_dict(), fa.flat_attn_tile_shape_get(128, 0).as_dict()
    assert (d64["rows_per_workgroup"], d64["wavefronts"], d64["lds_stages"]) == (256, 4, 4)
    assert (d128["rows_per_workgroup"], d128["wavefronts"], d128["lds_stages"]) == (256, 8, 3)


def test_cross_entry_point_validation():
    lib = fa.load_library()
    far = (0x1000, 1 << 40, 2 << 40, 3 << 40)

    def cross(Q=far[0], K=far[1], V=far[2], O=far[3], B=1, H=1, Nq=8, Nk=16, d=64, scale=1.0, mask=0, lens=None):
        return lib.flat_attn_fwd_cross(Q, K, V, O, B, H, Nq, Nk, d, scale, mask, lens, None)

    assert cross(Q=None) == -1 and cross(O=None) == -1
    assert cross(Nq=0) == -2 and cross(Nk=0) == -2 and cross(B=0) == -2
    assert cross(d=80) == -3 and cross(mask=3) == -3 and cross(scale=float("nan")) == -3
    assert cross(Nq=17, Nk=16, mask=1) == -3                 # causal: some query would see no key
    assert cross(K=far[1] + 4) == -4 and cross(lens=0x5002) == -4
    assert cross(O=far[1]) == -7 and cross(O=far[2] + 16) == -7
    assert cross(lens=far[3] + 16) == -7                      # the key counts may not live inside O
    assert cross(Nk=1 << 25, d=128) == -2 and cross(Nq=1 << 25, Nk=1 << 25, d=64) == -2


def test_blocksparse_entry_point_validation():
    lib = fa.load_library()
    far = (0x1000, 1 << 40, 2 << 40, 3 << 40)

    def sp(Q=far[0], K=far[1], V=far[2], O=far[3], B=1, H=1, N=512, d=64, scale=1.0, offs=0x9000, ids=0xA000, n=4):
        return lib.flat_attn_fwd_blocksparse(Q, K, V, O, B, H, N, d, scale, offs, ids, n, None)

    assert sp(Q=None) == -1 and sp(offs=None) == -1 and sp(ids=None) == -1
    assert sp(N=0) == -2 and sp(N=131072 + 1) == -2 and sp(n=-1) == -2
    assert sp(d=80) == -3 and sp(scale=-1.0) == -3
    assert sp(offs=0x9002) == -4 and sp(ids=0xA001) == -4 and sp(V=far[2] + 8) == -4
    assert sp(O=far[0]) == -7 and sp(offs=far[3] + 64) == -7 and sp(ids=far[3] + 128) == -7


def test_mix_probe_validation():
    lib = fa.load_probe_library()
    need_sink, need_src = fa.flat_attn_mix_probe_sink_bytes(), fa.flat_attn_mix_probe_src_bytes()
    assert need_sink == 512 * 256 * 4 and need_src == 2 * 64 * 8192
    assert fa.flat_attn_mix_probe_flops(1) == 512 * 4 * 8 * 16 * 32768.0 and fa.flat_attn_mix_probe_flops(0) == 0.0
    sink, src = 0x1000000, 0x8000000

    def probe(sink=sink, sink_bytes=need_sink, src=src, src_bytes=need_src, level=3, iters=4):
        return lib.flat_attn_mix_probe(sink, sink_bytes, src, src_bytes, level, iters, None)

    assert probe(sink=None) == -1 and probe(src=None) == -1
    assert probe(level=4) == -3 and probe(level=-1) == -3
    assert probe(iters=0) == -2 and probe(iters=(1 << 20) + 1) == -2
    assert probe(sink=sink + 4) == -4 and probe(src=src + 2) == -4
    assert probe(sink_bytes=need_sink - 1) == -5 and probe(src_bytes=need_src - 1) == -5
    assert probe(src=sink + 16) == -7


def test_streaming_asm_is_the_only_user_of_m0():
    """The global -> LDS loads are inline assembly that overwrites m0 without being able to declare it.  Compile the
    fused kernels to assembly and check that nothing else in them reads or writes m0."""
    import shutil
    import subprocess
    import tempfile
    from paper_2107_06419_amd import build as fb
    hipcc = fb._hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    src = os.path.join(ROOT, "paper_2107_06419_amd", "csrc", "flat_fwd_bf16.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        subprocess.run([hipcc, *fb.FLAGS, "-S", "--cuda-device-only", "-o", out, src], check=True, capture_output=True)
        inside, uses, dmas = False, [], 0
        for line in open(out):
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                inside = True
            elif t.startswith(";;#ASMEND"):
                inside = False
            elif re.search(r"\bm0\b", t.split(";")[0]):
                if inside:
                    dmas += "s_mov_b32 m0" in t
                else:
                    uses.append(t)
    assert dmas > 0, "no streaming load found: the check looks at the wrong file"
    assert not uses, f"m0 is used outside the streaming asm: {uses[:5]}"
