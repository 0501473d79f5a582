"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and its
argument validation / workspace planning behave as documented.  No GPU is needed (no compute calls)."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2510_25977_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def lib():
    if not B.LIB_PATH.exists():
        from paper_2510_25977_amd import build
        build.build(force=True)
    return B.lib()


def declared_symbols():
    text = (ROOT / "include" / "svdmlp.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svdmlp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    syms = declared_symbols()
    assert {"svdmlp_create", "svdmlp_forward", "svdmlp_destroy", "svdmlp_workspace_bytes"} <= set(syms)
    for s in syms:
        assert hasattr(lib, s), f"{s} declared in svdmlp.h but not exported"
    assert sorted(B.EXPORTS) == syms
    assert lib.svdmlp_abi_version() == 1


def desc(**kw):
    d = B.svdmlp_desc()
    d.kind, d.dtype = kw.get("kind", B.SVDMLP_GATED), kw.get("dtype", B.SVDMLP_BF16)
    d.max_M, d.d, d.ffn, d.r, d.r_down = kw.get("max_M", 64), kw.get("d", 256), kw.get("ffn", 512), kw.get("r", 128), kw.get("r_down", 128)
    for n in ("Ug", "Vg", "Uu", "Vu", "Ud", "Vd"):
        setattr(d, n, kw.get(n, 0x1000))
    d.workspace, d.workspace_bytes = kw.get("workspace", 0x100000), kw.get("workspace_bytes", 1 << 40)
    d.flags = kw.get("flags", B.FLAG_SKIP_ARCH_CHECK)
    return d


def create_status(d):
    out = ctypes.c_void_p()
    st = B.lib().svdmlp_create(ctypes.byref(d), ctypes.byref(out))
    if st == 0:
        B.lib().svdmlp_destroy(out)
    return st, out


def test_status_strings(lib):
    for code in (0, -1, -2, -3, -4, -5, -6, 17):
        s = lib.svdmlp_status_string(code)
        assert s and len(s) > 1
    assert b"workspace" in lib.svdmlp_status_string(B.SVDMLP_WORKSPACE_TOO_SMALL)


def test_workspace_bytes_formula(lib):
    d = desc(max_M=4096, d=4096, ffn=14336, r=512, r_down=512)
    n = B.svdmlp_workspace_bytes(d)
    factors = 2 * 3 * 512 * (4096 + 14336)
    assert n >= factors + 4096 * 1024 * 2          # re-tiled factors + rank-r strips
    assert n < factors + (400 << 20)
    # fp32: T [M,2r] + H [M,ffn] + Td [M,rd]
    d32 = desc(dtype=B.SVDMLP_F32, max_M=10, d=96, ffn=200, r=24, r_down=40)
    assert B.svdmlp_workspace_bytes(d32) >= 4 * 10 * (48 + 200 + 40)
    dl = desc(dtype=B.SVDMLP_F32, kind=B.SVDMLP_LINEAR, max_M=32, d=256, ffn=1024, r=16, r_down=0)
    assert 0 < B.svdmlp_workspace_bytes(dl) <= 4 * 32 * 16 + 256
    # bf16 LINEAR: re-tiled U and V + the rank-r strip of 256-row-padded M, the partial tiles of the first stage when it
    # cuts d (none at these extents), and the streaming path's 8 MiB of partial tiles and its ticket lines
    db = desc(kind=B.SVDMLP_LINEAR, max_M=300, d=512, ffn=1024, r=256, r_down=0)
    tickets = 32768 + 3 * 256 * 128 + 2 * 2048 * 128
    assert B.svdmlp_workspace_bytes(db) == 2 * (256 * 512 + 1024 * 256 + 512 * 256) + (8 << 20) + tickets


@pytest.mark.parametrize("kw,status", [
    (dict(max_M=0), B.SVDMLP_INVALID_ARGUMENT),
    (dict(d=-4), B.SVDMLP_INVALID_ARGUMENT),
    (dict(r=1024), B.SVDMLP_INVALID_ARGUMENT),                 # r > min(d, ffn)
    (dict(r_down=0), B.SVDMLP_INVALID_ARGUMENT),
    (dict(kind=7), B.SVDMLP_INVALID_ARGUMENT),
    (dict(dtype=9), B.SVDMLP_INVALID_ARGUMENT),
    (dict(Ug=0), B.SVDMLP_INVALID_ARGUMENT),                   # null factor
    (dict(Vd=0x1008), B.SVDMLP_INVALID_ARGUMENT),              # misaligned factor
    (dict(workspace=0), B.SVDMLP_INVALID_ARGUMENT),
    (dict(workspace=0x100010), B.SVDMLP_INVALID_ARGUMENT),     # workspace not 256-byte aligned
    (dict(workspace_bytes=1024), B.SVDMLP_WORKSPACE_TOO_SMALL),
    (dict(d=200), B.SVDMLP_UNSUPPORTED),                       # bf16 needs d % 128 == 0
    (dict(flags=B.FLAG_SKIP_ARCH_CHECK | B.FLAG_FORCE_TILED | B.FLAG_FORCE_STREAM), B.SVDMLP_INVALID_ARGUMENT),
])
def test_create_rejects_bad_descriptions(lib, kw, status):
    st, out = create_status(desc(**kw))
    assert st == status
    assert out.value is None                                   # *out is written only on success
    if status in (B.SVDMLP_INVALID_ARGUMENT, B.SVDMLP_UNSUPPORTED):
        if "workspace" not in kw and "Ug" not in kw and "Vd" not in kw:
            assert B.svdmlp_workspace_bytes(desc(**kw)) == 0


def test_host_only_context_lifecycle(lib):
    """With the architecture check skipped a context can be created without a device; forward then refuses."""
    out = ctypes.c_void_p()
    d = desc()
    assert lib.svdmlp_create(ctypes.byref(d), ctypes.byref(out)) == 0 and out.value
    assert lib.svdmlp_last_path(out) == 0 and lib.svdmlp_last_hip_error(out) == 0
    X, Y = ctypes.c_void_p(0x2000), ctypes.c_void_p(0x3000)
    assert lib.svdmlp_forward(out, X, 0, Y, None) == 0                                 # M = 0 is a no-op
    assert lib.svdmlp_forward(out, X, -1, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert lib.svdmlp_forward(out, X, 65, Y, None) == B.SVDMLP_INVALID_ARGUMENT        # M > max_M
    assert lib.svdmlp_forward(out, None, 4, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert lib.svdmlp_forward(out, X, 4, X, None) == B.SVDMLP_INVALID_ARGUMENT         # aliasing
    assert lib.svdmlp_forward(out, ctypes.c_void_p(0x2002), 4, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert lib.svdmlp_forward(out, X, 4, Y, None) == B.SVDMLP_NO_DEVICE               # nothing to run on
    assert lib.svdmlp_forward(None, X, 4, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    ms = (ctypes.c_float * 8)()
    nk, nf = ctypes.c_int(), ctypes.c_int()
    assert lib.svdmlp_profile_end(out, ms, ctypes.byref(nk), ctypes.byref(nf)) == B.SVDMLP_INVALID_ARGUMENT  # no profile open
    assert lib.svdmlp_profile_kernel_name(out, 0) is None
    assert lib.svdmlp_destroy(out) == 0
    assert lib.svdmlp_destroy(None) == 0


def test_static_scratch_forward_checks_its_arguments_without_a_device(lib):
    """The allocation-free variant validates like svdmlp_forward, takes only what streams (bf16, gated, up to 128 rows)
    and refuses extents whose per-forward buffers pass the static array, all before touching a device."""
    assert lib.svdmlp_static_scratch_bytes() == 16 << 20
    fwd = lib.svdmlp_forward_static_scratch
    X, Y = ctypes.c_void_p(0x2000), ctypes.c_void_p(0x3000)
    out = ctypes.c_void_p()
    d = desc(max_M=300)
    assert lib.svdmlp_create(ctypes.byref(d), ctypes.byref(out)) == 0
    assert fwd(out, X, 0, Y, None) == 0
    assert fwd(out, X, -1, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert fwd(out, X, 301, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert fwd(out, None, 4, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert fwd(out, X, 4, X, None) == B.SVDMLP_INVALID_ARGUMENT
    assert fwd(out, ctypes.c_void_p(0x2002), 4, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert fwd(None, X, 4, Y, None) == B.SVDMLP_INVALID_ARGUMENT
    assert fwd(out, X, 129, Y, None) == B.SVDMLP_UNSUPPORTED          # beyond the weight-streaming path
    assert fwd(out, X, 128, Y, None) == B.SVDMLP_NO_DEVICE            # would run: host-only context
    lib.svdmlp_destroy(out)
    for kw in (dict(dtype=B.SVDMLP_F32), dict(kind=B.SVDMLP_LINEAR)):
        d = desc(**kw)
        assert lib.svdmlp_create(ctypes.byref(d), ctypes.byref(out)) == 0
        assert fwd(out, X, 4, Y, None) == B.SVDMLP_UNSUPPORTED
        lib.svdmlp_destroy(out)
    # 128 rows x ffn = 30720: the activation alone is 7.9 MB, the array has 7.5 MiB for T, H and Td
    d = desc(max_M=128, ffn=30720)
    assert lib.svdmlp_create(ctypes.byref(d), ctypes.byref(out)) == 0
    assert fwd(out, X, 128, Y, None) == B.SVDMLP_SCRATCH_TOO_SMALL
    assert fwd(out, X, 65, Y, None) == B.SVDMLP_SCRATCH_TOO_SMALL     # 65 rows run as 128
    assert fwd(out, X, 64, Y, None) == B.SVDMLP_NO_DEVICE             # fits
    assert b"static scratch" in lib.svdmlp_status_string(B.SVDMLP_SCRATCH_TOO_SMALL)
    lib.svdmlp_destroy(out)


def test_force_plan_checks_its_arguments_and_plan_room_grows_the_workspace(lib):
    out = ctypes.c_void_p()
    d = desc(max_M=4096, d=4096, ffn=14336, r=512, r_down=512)
    assert lib.svdmlp_create(ctypes.byref(d), ctypes.byref(out)) == 0
    fp = lib.svdmlp_force_plan
    assert fp(out, 0, 0, 0, 0) == 0 and fp(out, B.FIRST_IN, 4, 16, B.OUT_128) == 0 and fp(out, B.FIRST_S1, 0, 0, 0) == 0
    for bad in ((3, 0, 0, 0), (-1, 0, 0, 0), (1, 9, 0, 0), (0, 2, 0, 0), (0, 0, 33, 0), (0, 0, -1, 0), (0, 0, 0, 3)):
        assert fp(out, *bad) == B.SVDMLP_INVALID_ARGUMENT, bad
    assert fp(None, 0, 0, 0, 0) == B.SVDMLP_INVALID_ARGUMENT
    lib.svdmlp_destroy(out)
    d32 = desc(dtype=B.SVDMLP_F32)
    assert lib.svdmlp_create(ctypes.byref(d32), ctypes.byref(out)) == 0
    assert fp(out, 0, 0, 4, 0) == B.SVDMLP_UNSUPPORTED
    lib.svdmlp_destroy(out)
    # room for every candidate: 32 ranges of the down projection's partial sums instead of the planner's 8
    plain = B.svdmlp_workspace_bytes(d)
    d.flags |= B.FLAG_PLAN_ROOM
    roomy = B.svdmlp_workspace_bytes(d)
    assert 20 * 4096 * 512 * 4 <= roomy - plain <= 24 * 4096 * 512 * 4


def test_small_batches_fall_back_to_the_tiled_path_when_the_streaming_path_has_no_room():
    """The weight-streaming path has 2048 ticket lines per split phase; a context whose rank needs more (beyond 32768)
    is still legal, and its small batches take the MFMA-tiled path instead of failing at the first forward."""
    big = desc(max_M=128, d=65536, ffn=65536, r=40960, r_down=40960)
    for M in (1, 16, 33, 128):
        assert plan_of(big, M).startswith("path=5"), M
    big.flags |= B.FLAG_FORCE_STREAM
    with pytest.raises(B.SvdMlpError) as e:
        B.svdmlp_describe(big, 16)
    assert e.value.status == B.SVDMLP_UNSUPPORTED
    ok = desc(max_M=128, d=65536, ffn=65536, r=16384, r_down=16384)
    assert plan_of(ok, 16).startswith("path=3") and plan_of(ok, 128).startswith("path=3")


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", tmp_path / "nope.so")
    with pytest.raises(FileNotFoundError):
        B.lib()


def plan_of(d, M):
    """The plan description without the cost model's figures (est_us and the alternatives of a stage)."""
    return re.sub(r" est_us=[^\]]*", "", B.svdmlp_describe(d, M))


def test_describe_prints_the_cost_model_scores_of_each_stage():
    """Every stage that leaves a choice shows the estimated time of the chosen candidate and of the closest others,
    and the chosen one is the cheapest the model lists (the choice is made by the model, not by a rule beside it)."""
    pre = desc(max_M=4096, d=4096, ffn=14336, r=512, r_down=512)
    s = B.svdmlp_describe(pre, 4096)
    stages = re.findall(r"(k_s1|k_in|k_down1|k_out|k_s5)\[[^\]]*? est_us=([0-9.]+) alternatives:([^\]]*)\]", s)
    assert [k for k, _, _ in stages] == ["k_s1", "k_down1", "k_out"], s
    for kernel, est, alts in stages:
        others = [float(x.split("=")[1]) for x in alts.split()]
        assert others, (kernel, s)
        assert float(est) <= min(others), (kernel, s)
    # the first stage weighs both kernels and several cuts of the contraction
    first_alts = stages[0][2]
    assert "in/" in first_alts and "s1/2=" in first_alts
    assert "out128/1=" in stages[2][2]


def test_describe_names_the_plan_of_every_baseline_config():
    """svdmlp_describe is host-only: the planner's choices for the BASELINE configurations, pinned so that a change
    of the cost model shows up here (tile shapes, contraction ranges, persistent workgroups, half-tile round)."""
    pre = desc(max_M=4096, d=4096, ffn=14336, r=512, r_down=512)
    s = plan_of(pre, 4096)
    assert s.startswith("path=5 bf16-tiled-staged:")
    assert "k_s1[tile=128x128 tiles=256 ranges=1]" in s
    assert "k_gate_up[tile=256x256 tiles=896 workgroups=256 full=768 halves=256 xcd_grid=4x2]" in s
    assert "k_down1[tile=256x256 tiles=32 ranges=8] k_reduce k_out[tile=256x256 tiles=256]" in s
    # decode shape: one row tile, both split phases fill the chip, and so does the last product on 16-column tiles
    s = plan_of(pre, 16)
    assert s.startswith("path=3 bf16-streaming: row_tiles=1 k_stream_d1[tile=16 tiles=64 ranges=4] k_stream_d2[tiles=448]")
    assert "k_stream_d4[tile=16 tiles=32 ranges=8] k_stream_d5[tile=16 tiles=256]" in s
    assert plan_of(pre, 32) == s
    # two row tiles: 32-column tiles, each row tile with workgroups of its own in the two cut phases and in the last one
    s = plan_of(pre, 33)
    assert s.startswith("path=3 bf16-streaming: row_tiles=2 k_stream_d1[tiles=32 row_groups=2 ranges=4] k_stream_d2[tiles=448]")
    assert "k_stream_d4[tiles=16 row_groups=2 ranges=8] k_stream_d5[tiles=128 row_groups=2]" in s
    assert plan_of(pre, 64) == s
    # four row tiles: 8 MB of [Ug|Uu] are worth fetching four times to shorten the partial sums' read-back, 15 MB of Ud twice
    s = plan_of(pre, 128)
    assert s.startswith("path=3 bf16-streaming: row_tiles=4 k_stream_d1[tiles=32 row_groups=4 ranges=2] k_stream_d2[tiles=448]")
    assert "k_stream_d4[tiles=16 row_groups=2 ranges=8] k_stream_d5[tiles=128 row_groups=2]" in s
    assert plan_of(pre, 129).startswith("path=5")
    # config 2 (M = 128) streams, small factors: row-tile groups in every phase that has too few tiles;
    # forced onto the tiled path it has one row tile
    small = desc(max_M=128, d=2048, ffn=8192, r=256, r_down=256)
    s = plan_of(small, 128)
    assert s.startswith("path=3 bf16-streaming: row_tiles=4 k_stream_d1[tiles=16 row_groups=4 ranges=4] k_stream_d2[tiles=256]")
    assert "k_stream_d4[tiles=8 row_groups=4 ranges=8] k_stream_d5[tiles=64 row_groups=4]" in s
    small.flags |= B.FLAG_FORCE_TILED
    # fewer tiles than half the CUs: every tile of k_gate_up as two 128-row halves
    assert "k_gate_up[tile=256x256 tiles=32 workgroups=32 full=0 halves=64" in plan_of(small, 128)
    # wide config: 8 row tiles x 108 column tiles = 3 full rounds + 96 tiles as 192 halves
    wide = desc(max_M=2048, d=5120, ffn=27648, r=1024, r_down=1024)
    s = plan_of(wide, 2048)
    assert "k_gate_up[tile=256x256 tiles=864 workgroups=256 full=768 halves=192" in s
    # fused variant on request, and for extents the staged one does not take
    pre.flags |= B.FLAG_TILED_FUSED
    assert plan_of(pre, 4096).startswith("path=2 bf16-tiled-fused:")
    odd = desc(max_M=512, d=256, ffn=384, r=192, r_down=128)   # ffn and r_down run rounded up to 512 and 256
    assert plan_of(odd, 512).startswith("path=5")
    # both ranks within one 128-wide tile: the fused variant by itself (the staged one would pad r_down to 256 and is
    # bound by the round trip of the activation at so little arithmetic per element)
    tiny = desc(max_M=4096, d=4096, ffn=14336, r=128, r_down=128)
    assert plan_of(tiny, 4096).startswith("path=2 bf16-tiled-fused:")
    assert "k_stream_d4[tile=16 tiles=8 " in plan_of(tiny, 16)      # the streaming path runs r_down = 128 unpadded
    # single factored layer at the paper's kernel-evaluation shape: the first stage cuts d when tiles are few
    lin = desc(kind=B.SVDMLP_LINEAR, max_M=32768, d=8192, ffn=16384, r=4096, r_down=0)
    assert "k_in[tile=256x256 tiles=64 ranges=4] k_reduce k_out" in plan_of(lin, 1024)
    assert "k_in[tile=256x256 tiles=256 ranges=1] k_out[tile=256x256 tiles=1024]" in plan_of(lin, 4096)
    # up to 128 rows the layer streams its weights (phases D1 and D5 of the streaming path), unless re-reading the
    # activation for every weight tile would cost more than the tiles (this shape beyond 64 rows)
    assert plan_of(lin, 16).startswith("path=7 bf16-linear-streaming: row_tiles=1 k_stream_d1[tile=16 tiles=256 ranges=1] k_stream_d5[tiles=512")
    assert plan_of(lin, 64).startswith("path=7") and plan_of(lin, 65).startswith("path=6")
    assert plan_of(desc(kind=B.SVDMLP_LINEAR, max_M=128, d=4096, ffn=4096, r=1024, r_down=0), 128).startswith("path=7")
    # the small-block point of the block-size comparison: both products on 128 x 128 tiles on request
    lin.flags |= B.FLAG_TILE_128
    assert "k_s1[tile=128x128 tiles=1024 ranges=1] k_s5[tile=128x128 tiles=4096]" in plan_of(lin, 4096)
    f32 = desc(dtype=B.SVDMLP_F32, max_M=10, d=96, ffn=200, r=24, r_down=40)
    assert plan_of(f32, 10).startswith("path=1")
    # errors
    with pytest.raises(B.SvdMlpError) as e:
        B.svdmlp_describe(pre, 5000)
    assert e.value.status == B.SVDMLP_INVALID_ARGUMENT
    with pytest.raises(B.SvdMlpError) as e:
        B.svdmlp_describe(desc(d=200), 8)
    assert e.value.status == B.SVDMLP_UNSUPPORTED


def test_ranks_are_rounded_up_to_the_tiles():
    """Any rank up to min(d, ffn) is accepted on the bf16 path: the plan runs with the rank rounded up (zero columns /
    rows in the re-tiled factors), which shows in the workspace size and in the plan description."""
    base = B.svdmlp_workspace_bytes(desc(max_M=300, d=1024, ffn=1024, r=256, r_down=768))
    for r, rd in ((200, 768), (256, 600), (193, 513)):
        assert B.svdmlp_workspace_bytes(desc(max_M=300, d=1024, ffn=1024, r=r, r_down=rd)) == base, (r, rd)
    assert B.svdmlp_workspace_bytes(desc(max_M=300, d=1024, ffn=1024, r=257, r_down=768)) > base
    # staged variant: down rank to a multiple of 256; fused variant (on request, or ffn not a multiple of 256): to 128, 256,
    # 512 or a multiple of 512
    assert "k_down1[tile=256x256 tiles=6 ranges" in plan_of(desc(max_M=300, d=1024, ffn=1024, r=200, r_down=600), 300)
    # ffn is internal to the gated forward: rounded up to a multiple of 256 as well (1100 -> 1280 = 5 column tiles)
    s = plan_of(desc(max_M=300, d=1024, ffn=1100, r=200, r_down=600), 300)
    assert s.startswith("path=5 bf16-tiled-staged:") and "k_gate_up[tile=256x256 tiles=10 " in s
    fused = desc(max_M=300, d=1024, ffn=1100, r=200, r_down=600)
    fused.flags |= B.FLAG_TILED_FUSED
    assert plan_of(fused, 300).startswith("path=2 bf16-tiled-fused:")
    lin = desc(kind=B.SVDMLP_LINEAR, max_M=300, d=512, ffn=640, r=100, r_down=0)
    assert B.svdmlp_workspace_bytes(lin) == B.svdmlp_workspace_bytes(desc(kind=B.SVDMLP_LINEAR, max_M=300, d=512, ffn=640, r=128, r_down=0))


def test_header_is_plain_c_and_a_c_program_links(lib, tmp_path):
    """include/svdmlp.h compiles as C99 with gcc, and a C caller can use the host-only entry points."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "svdmlp.h"
int main(void) {
  svdmlp_desc de;
  memset(&de, 0, sizeof de);
  de.kind = SVDMLP_GATED; de.dtype = SVDMLP_BF16;
  de.max_M = 4096; de.d = 4096; de.ffn = 14336; de.r = 512; de.r_down = 512;
  de.flags = SVDMLP_FLAG_SKIP_ARCH_CHECK;
  char line[1024];
  if (svdmlp_describe(&de, 4096, line, sizeof line) != SVDMLP_OK) return 1;
  printf("%d %zu %s\n", svdmlp_abi_version(), svdmlp_workspace_bytes(&de), line);
  return svdmlp_destroy(NULL);
}
''')
    exe = tmp_path / "use"
    libdir = B.LIB_PATH.parent
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", str(ROOT / "include"), str(src), "-o", str(exe),
                    "-L", str(libdir), "-lsvdmlp", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(" ", 2)
    assert int(out[0]) == 1 and int(out[1]) > 0 and out[2].startswith("path=5 bf16-tiled-staged:")


def test_rank_for_ratio_follows_the_rank_rule():
    """svdmlp_rank_for_ratio (paper Eq. 5): hand-evaluated cases, the never-zero rule, argument checks, and agreement
    with the Python cost model over a grid of layer shapes and ratios."""
    from paper_2510_25977_amd import costmodel as cm
    # 2048*8192*0.8/(10240*128) = 10.24 -> floor(10.74) = 10 blocks; 4096*14336*0.95/(18432*128) = 23.64 -> 24 blocks
    assert B.svdmlp_rank_for_ratio(2048, 8192, 0.2, 128, 0.5) == 1280
    assert B.svdmlp_rank_for_ratio(4096, 14336, 0.05, 128, 0.5) == 3072
    assert B.svdmlp_rank_for_ratio(4096, 14336, 0.05, 128, 0.0) == 23 * 128      # alpha = 0: round down
    assert B.svdmlp_rank_for_ratio(64, 64, 0.99, 128, 0.5) == 128                # at least one block
    for k, n in [(2048, 8192), (4096, 14336), (5120, 27648), (7168, 18432), (48, 80)]:
        for ratio in (0.0, 0.1, 0.2, 0.35, 0.5, 0.8, 0.95):
            for block in (8, 128, 256):
                assert B.svdmlp_rank_for_ratio(k, n, ratio, block, 0.5) == cm.block_aligned_rank(k, n, ratio, block)
    for bad in [(0, 8, 0.1, 128, 0.5), (8, -1, 0.1, 128, 0.5), (8, 8, 1.0, 128, 0.5), (8, 8, -0.1, 128, 0.5), (8, 8, 0.1, 0, 0.5),
                (8, 8, 0.1, 128, 1.5), (8, 8, float("nan"), 128, 0.5)]:
        assert B.lib().svdmlp_rank_for_ratio(*bad) == -1


def test_build_step_catches_an_sgpr_written_by_a_vector_instruction_right_before_a_handwritten_store():
    """The hand-written copies and stores take their base address in SGPRs inside an asm statement, where the compiler
    cannot see the five wait states that a vector-written SGPR needs before a memory instruction reads it.  The build
    checks the generated assembly; this pins the checker on the pattern that once faulted (a spilled SGPR restored by
    v_readlane directly before the store) and on the variants that are fine."""
    from paper_2510_25977_amd import build as bld
    bad = """
	v_cvt_pk_bf16_f32 v83, v83, v84
	v_readlane_b32 s5, v245, 2
	;;#ASMSTART
	global_store_dwordx4 v240, v[80:83], s[4:5] nt
	s_nop 1
	;;#ASMEND
"""
    assert len(bld.check_sgpr_hazards(bad)) == 1
    # five wait states in between (s_nop 3 = four, plus one other instruction): fine
    assert bld.check_sgpr_hazards(bad.replace(";;#ASMSTART", "s_nop 3\n\tv_mov_b32 v1, v2\n\t;;#ASMSTART")) == []
    # four are not enough
    assert len(bld.check_sgpr_hazards(bad.replace(";;#ASMSTART", "s_nop 3\n\t;;#ASMSTART"))) == 1
    # another register, a scalar write, or the compiler's own store (outside an asm statement) are not findings
    assert bld.check_sgpr_hazards(bad.replace("s5, v245", "s7, v245")) == []
    assert bld.check_sgpr_hazards(bad.replace("v_readlane_b32 s5, v245, 2", "s_add_u32 s5, s5, 1")) == []
    assert bld.check_sgpr_hazards(bad.replace(";;#ASMSTART", "").replace(";;#ASMEND", "")) == []
    # the copy into LDS: its own s_mov / s_nop count as two of the five
    dma = """
	v_readfirstlane_b32 s34, v3
	s_add_i32 s9, s9, 1
	s_add_i32 s9, s9, 1
	;;#ASMSTART
	s_mov_b32 m0, s96
	s_nop 0
	global_load_lds_dwordx4 v240, s[34:35]
	;;#ASMEND
"""
    assert len(bld.check_sgpr_hazards(dma)) == 1
    assert bld.check_sgpr_hazards(dma.replace("s_add_i32 s9, s9, 1\n\ts_add_i32 s9, s9, 1", "s_nop 2")) == []


def test_roof_entry_points_reject_bad_arguments_before_any_launch(lib):
    """The roof microbenchmarks validate their arguments on the host: nothing is enqueued for a null sink, a count
    that is not positive, an operand set outside 0..2, more than 1024 threads or a misaligned buffer."""
    sink, buf = ctypes.c_void_p(0x4000), ctypes.c_void_p(0x10000)
    bad = B.SVDMLP_INVALID_ARGUMENT
    for fn in (lib.svdmlp_roof_mfma_operands, lib.svdmlp_roof_pingpong):
        fn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        assert fn(0, 1, sink, 4, None) == bad
        assert fn(8, 3, sink, 4, None) == bad
        assert fn(8, -1, sink, 4, None) == bad
        assert fn(8, 1, None, 4, None) == bad
        assert fn(8, 1, sink, 0, None) == bad
    lib.svdmlp_roof_mfma.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    assert lib.svdmlp_roof_mfma(0, sink, 4, None) == bad
    assert lib.svdmlp_roof_mfma(8, None, 4, None) == bad
    lib.svdmlp_roof_coexec.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    assert lib.svdmlp_roof_coexec(-1, 1, sink, 4, None) == bad
    assert lib.svdmlp_roof_coexec(1, 1, None, 4, None) == bad
    lib.svdmlp_roof_empty.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    assert lib.svdmlp_roof_empty(0, 64, None) == bad
    assert lib.svdmlp_roof_empty(4, 2048, None) == bad
    lib.svdmlp_roof_empty_chain.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    assert lib.svdmlp_roof_empty_chain(0, 4, 64, None) == bad
    assert lib.svdmlp_roof_empty_chain(4, 4, 0, None) == bad
    lib.svdmlp_roof_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    assert lib.svdmlp_roof_read(None, 1 << 20, sink, 4, None) == bad
    assert lib.svdmlp_roof_read(buf, 1024, sink, 4, None) == bad                       # less than one block
    assert lib.svdmlp_roof_read(ctypes.c_void_p(0x10004), 1 << 20, sink, 4, None) == bad   # not 16-byte aligned
    assert lib.svdmlp_roof_read(buf, 1 << 20, None, 4, None) == bad
