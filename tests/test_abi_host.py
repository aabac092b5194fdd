"""Host-only checks of the C-ABI library: it loads, exports every symbol the header
declares, sizes its workspace without an N*V term, and rejects bad arguments before
touching any device."""
import ctypes
import os
import re

import pytest

from paper_2511_17599_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flce.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flce_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert re.fullmatch(r"\d+\.\d+\.\d+", B.flce_version())
    assert B.flce_status_string(B.FLCE_OK) == "ok"
    assert "target" in B.flce_status_string(B.FLCE_ERR_TARGET_RANGE)


def plan_fields(N, d, V, dt):
    text = B.flce_plan_describe(N, d, V, dt)
    return text, {k: v for k, v in (t.split("=") for t in text.split() if "=" in t)}


def test_workspace_beyond_the_staging_cap_has_no_NV_term():
    for dt in (B.FLCE_DTYPE_BF16, B.FLCE_DTYPE_F32):
        for bwd in (0, 1):
            base = B.flce_workspace_bytes(8192, 4096, 128256, dt, bwd)
            assert base > 0
            # doubling N and V together would quadruple an N*V term; the workspace at most ~doubles
            big = B.flce_workspace_bytes(16384, 4096, 256512, dt, bwd)
            assert big <= 2.2 * base + (1 << 20)
    # the long-sequence shape: naive fp32 logits are 67 GB, the workspace stays far below that
    ws = B.flce_workspace_bytes(131072, 4096, 128256, B.FLCE_DTYPE_BF16, 1)
    assert ws < 0.12 * 131072 * 128256 * 4
    fw = B.flce_workspace_bytes(131072, 4096, 128256, B.FLCE_DTYPE_BF16, 0)
    assert fw < 131072 * 4096 * 2 + 64 * (1 << 20)          # at most one copy of H plus per-row partials
    # staging never exceeds its cap however large the problem
    for N, V in ((131072, 128256), (1 << 20, 1 << 20), (600000, 600), (600, 600000)):
        _, f = plan_fields(N, 4096, V, B.FLCE_DTYPE_BF16)
        assert int(f["staging_bytes"]) <= 32768 * (32768 + 64) * 2


def test_workspace_below_the_staging_cap_is_what_the_header_says():
    """A problem smaller than the staging cap stages its whole G (storage type): that part does grow like N x V,
    everything else like (N + V) d.  Checked at a shape under the cap, at the same shape doubled, and at the tiny
    fp32 benchmark shape (generic loop: transposed copies on top)."""
    dt, e = B.FLCE_DTYPE_BF16, 2

    def parts(N, d, V):
        _, f = plan_fields(N, d, V, dt)
        staging, total = int(f["staging_bytes"]), int(f["bwd_ws"])
        assert total == B.flce_workspace_bytes(N, d, V, dt, 1)
        return staging, total - staging

    s1, r1 = parts(4096, 768, 16384)
    s2, r2 = parts(8192, 768, 32768)
    assert s1 == 4096 * (16384 + 64) * e and s2 == 8192 * (32768 + 64) * e      # the whole (padded) G
    assert 3.9 < s2 / s1 < 4.1                                                    # that part is N x V
    # the rest is (N + V) d: copies of H, fp32 running sums, at most 8 fp32 K-slice tiles of the larger output
    for (N, d, V), rest in (((4096, 768, 16384), r1), ((8192, 768, 32768), r2)):
        assert rest <= 2 * N * d * e + 16 * N + 4 * N * d + 4 * V * d + 8 * 4 * max(N, V) * d + (1 << 20)
    # the bf16 staging is half the fp32 logits it replaces; with the other buffers the backward stays below them
    assert B.flce_workspace_bytes(4096, 768, 50257, dt, 1) < 0.62 * 4096 * 50257 * 4
    # tiny fp32 shape (generic loop): G, its transpose, a transposed W chunk and 8 K-slice tiles of dH
    text, f = plan_fields(256, 256, 4096, B.FLCE_DTYPE_F32)
    assert "loop=generic" in text
    tiny = int(f["bwd_ws"])
    assert tiny <= 4 * 256 * (4096 + 64) * 4 and tiny > 256 * 4096 * 4            # several times the 4 MB of logits
    assert int(f["fwd_ws"]) < 64 * 1024


def test_static_scratch_limit_is_checked_on_the_host():
    p = 4096
    assert B.flce_forward_static(p, p, p, 400000, 4096, 128256, -100, B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_BF16, p, p) == \
        B.FLCE_ERR_WORKSPACE
    assert B.flce_forward_static(None, p, p, 256, 64, 512, -100, B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_BF16, p, p) == \
        B.FLCE_ERR_BAD_ARG


def test_probe_and_plan_reject_bad_shapes_on_the_host():
    p = 4096
    assert B.flce_probe(0, p, p, p, 256, 256, 31, 4, 1, p) == B.FLCE_ERR_BAD_SHAPE       # K not a multiple of 32
    assert B.flce_probe(0, p, p, p, 250, 256, 64, 4, 1, p) == B.FLCE_ERR_BAD_SHAPE       # rows not whole tiles
    assert B.flce_probe(len(B.PROBE_MODES), p, p, p, 256, 256, 64, 4, 1, p) == B.FLCE_ERR_BAD_ARG   # unknown mode
    assert B.flce_probe(0, None, p, p, 256, 256, 64, 4, 1, p) == B.FLCE_ERR_BAD_ARG
    with pytest.raises(ValueError):
        B.flce_plan_describe(64, 60, 64, B.FLCE_DTYPE_BF16)
    assert "windows=" in B.flce_plan_describe(64, 64, 64, B.FLCE_DTYPE_BF16)


def _plan(N, d, V):
    return dict(kv.split("=") for kv in B.flce_plan_describe(N, d, V, B.FLCE_DTYPE_BF16).split()[2:])


def test_k_split_tails_are_planned_where_a_last_round_is_mostly_empty():
    """A contraction launch of one to four rounds of 256 output tiles with a last round less than half full gets a
    K-split tail (output-row tiles x slices); its slices fill at most one round and cost at most 64 MiB."""
    # GPT-2 shape: dW has 197 x 3 = 591 tiles: 170 row tiles whole (510 tiles), 27 in 3 slices (243 workgroups)
    assert _plan(4096, 768, 50257)["tail_dW"] == "27x3"
    # Llama shape: dW 128 x 16 = 2048 tiles = 8 rounds (none: too many rounds), dH 32 x 16 = 2 rounds exactly
    p = _plan(8192, 4096, 128256)
    assert p["tail_dW"] == "0x1" and p["tail_dH"] == "0x1"
    # a launch that is K-split as a whole has no tail on top
    p = _plan(8192, 3072, 256000)
    assert p["splitk_dH"] == "2" and p["tail_dH"] == "0x1"
    for N, d, V in [(1024, 768, 23040), (5120, 3584, 2048), (4096, 768, 50257), (2048, 1024, 40000), (3072, 512, 70000)]:
        p = _plan(N, d, V)
        n_mt = -(-d // 256)
        for key in ("tail_dH", "tail_dW"):
            rows, slices = map(int, p[key].split("x"))
            if rows:
                assert slices >= 2 and rows * n_mt * slices <= 256
                assert slices * rows * 256 * d * 4 <= 64 << 20


@pytest.mark.parametrize("N,d,V", [(0, 64, 64), (64, 0, 64), (64, 64, 0), (64, 60, 64), (-1, 64, 64)])
def test_bad_shapes_are_rejected(N, d, V):
    assert B.flce_workspace_bytes(N, d, V, B.FLCE_DTYPE_BF16, 0) == 0
    st = B.flce_forward(256, 256, 256, N, d, V, -100, B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_BF16, 256, 256, 256, 1 << 30)
    assert st == B.FLCE_ERR_BAD_SHAPE


def test_bad_arguments_are_rejected_without_a_device():
    ok = dict(N=256, d=64, V=512)
    need_f = B.flce_workspace_bytes(256, 64, 512, B.FLCE_DTYPE_F32, 0)
    need_b = B.flce_workspace_bytes(256, 64, 512, B.FLCE_DTYPE_F32, 1)
    p = 4096  # a fake, aligned, never dereferenced device address
    f = lambda **kw: B.flce_forward(kw.get("H", p), p, p, ok["N"], ok["d"], ok["V"], -100,
                                    kw.get("red", B.FLCE_REDUCE_MEAN), kw.get("dt", B.FLCE_DTYPE_F32), p, p,
                                    kw.get("ws", p), kw.get("wsb", need_f))
    assert f(H=None) == B.FLCE_ERR_BAD_ARG
    assert f(H=p + 4) == B.FLCE_ERR_BAD_ARG                 # misaligned tensor
    assert f(red=2) == B.FLCE_ERR_BAD_ARG
    assert f(dt=7) == B.FLCE_ERR_BAD_ARG
    assert f(ws=None) == B.FLCE_ERR_WORKSPACE
    assert f(ws=p + 16) == B.FLCE_ERR_WORKSPACE             # misaligned workspace
    assert f(wsb=need_f - 1) == B.FLCE_ERR_WORKSPACE
    b = lambda **kw: B.flce_backward(p, p, p, kw.get("lse", p), 256, 64, 512, -100, B.FLCE_REDUCE_SUM,
                                     B.FLCE_DTYPE_F32, 1.0, p, kw.get("dW", p), p, kw.get("wsb", need_b))
    assert b(lse=None) == B.FLCE_ERR_BAD_ARG
    assert b(dW=None) == B.FLCE_ERR_BAD_ARG
    assert b(wsb=need_b - 1) == B.FLCE_ERR_WORKSPACE
    assert B.lib().flce_last_device_status(None, None, None) == B.FLCE_ERR_BAD_ARG
    # Alg. 3 / Alg. 4 entry points: one workspace that serves both halves, no NULL tensors
    g = lambda **kw: B.flce_forward_with_grads(p, p, p, 256, 64, 512, -100, B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_F32, p, p,
                                               kw.get("dH", p), p, p, kw.get("wsb", max(need_f, need_b)))
    assert g(dH=None) == B.FLCE_ERR_BAD_ARG
    assert g(wsb=max(need_f, need_b) - 1) == B.FLCE_ERR_WORKSPACE
    sc = lambda **kw: B.flce_scale(p, kw.get("dWp", p), 256, kw.get("d", 64), 512, kw.get("red", B.FLCE_REDUCE_MEAN),
                                   B.FLCE_DTYPE_F32, 1.0, kw.get("ws", p), p, p)
    assert sc(dWp=None) == B.FLCE_ERR_BAD_ARG
    assert sc(ws=None) == B.FLCE_ERR_BAD_ARG
    assert sc(red=5) == B.FLCE_ERR_BAD_ARG
    assert sc(d=63) == B.FLCE_ERR_BAD_SHAPE
    # vocabulary-sliced calls: the slice must lie inside [0, V_total); the merge needs its own small workspace
    fp = lambda **kw: B.flce_forward_partial(p, p, p, 256, 64, kw.get("Vs", 128), kw.get("v0", 384), 512, -100,
                                             B.FLCE_DTYPE_F32, kw.get("m", p), p, p, p, kw.get("wsb", need_f))
    assert fp(v0=385) == B.FLCE_ERR_BAD_SHAPE
    assert fp(v0=-1) == B.FLCE_ERR_BAD_SHAPE
    assert fp(m=None) == B.FLCE_ERR_BAD_ARG
    assert fp(wsb=16) == B.FLCE_ERR_WORKSPACE
    need_m = B.flce_merge_workspace_bytes(256)
    assert 0 < need_m <= 4096 and B.flce_merge_workspace_bytes(0) == 0
    mp = lambda **kw: B.flce_merge_partials(p, kw.get("a", p), p, kw.get("n", 2), p, 256, 512, -100,
                                            B.FLCE_REDUCE_MEAN, p, p, p, kw.get("wsb", need_m))
    assert mp(a=None) == B.FLCE_ERR_BAD_ARG
    assert mp(n=0) == B.FLCE_ERR_BAD_ARG
    assert mp(wsb=need_m - 1) == B.FLCE_ERR_WORKSPACE
    bp = lambda **kw: B.flce_backward_partial(p, p, p, p, 256, 64, 128, kw.get("v0", 0), kw.get("Vt", 512), -100,
                                              B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_F32, 1.0, p, kw.get("dW", p), p,
                                              kw.get("wsb", need_b))
    assert bp(Vt=100) == B.FLCE_ERR_BAD_SHAPE
    assert bp(dW=None) == B.FLCE_ERR_BAD_ARG
    assert bp(wsb=16) == B.FLCE_ERR_WORKSPACE
    # per-row variant: label smoothing must lie in [0, 1); the per-row arrays must be there
    fr = lambda **kw: B.flce_forward_rows(p, p, p, 256, 64, 512, -100, kw.get("eps", 0.1), B.FLCE_DTYPE_F32,
                                          kw.get("rows", p), p, p, need_f)
    assert fr(eps=1.0) == B.FLCE_ERR_BAD_ARG
    assert fr(eps=-0.1) == B.FLCE_ERR_BAD_ARG
    assert fr(eps=float("nan")) == B.FLCE_ERR_BAD_ARG
    assert fr(rows=None) == B.FLCE_ERR_BAD_ARG
    br = lambda **kw: B.flce_backward_rows(p, p, p, p, kw.get("g", p), 256, 64, 512, -100, kw.get("eps", 0.0),
                                           B.FLCE_DTYPE_F32, p, p, p, kw.get("wsb", need_b))
    assert br(g=None) == B.FLCE_ERR_BAD_ARG
    assert br(eps=1.5) == B.FLCE_ERR_BAD_ARG
    assert br(wsb=need_b - 1) == B.FLCE_ERR_WORKSPACE


def test_header_is_plain_c(tmp_path):
    """The boundary header compiles as C99 on its own (no C++ or HIP types in the signatures)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_flce.c"
    src.write_text('#include "flce.h"\nint main(void) { flce_status (*f)(int) = flce_profile_enable; return f == 0 ? FLCE_PROF_CLASSES : FLCE_OK; }\n')
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
