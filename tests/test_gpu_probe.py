"""The measurement probe's main-loop modes compute real products: every thread's sink value is the sum, over the
tiles its workgroup walked, of one known accumulator element per 32x32 block, so it can be checked against a plain
matrix product.  (The figures the probe is used for would mean little if the loops it times moved the wrong data.)"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2511_17599_amd import binding as B             # noqa: E402


@pytest.fixture(autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _expected(C, mode_name, wgs, tiles, a_rows, b_rows):
    """sink[wg][thread] from the product C = A.B^T, following the probe's tile walk and accumulator layout."""
    half = mode_name.startswith("half")
    AM, a_tile = (2, 128) if half else (4, 256)
    n_bt, n_at = b_rows // 256, a_rows // a_tile
    tid = np.arange(256)
    wave, lane = tid >> 6, tid & 63
    exp = np.zeros((wgs, 256))
    for blk in range(wgs):
        b0 = (blk % n_bt) * 256
        for t in range(tiles):
            first = (blk // n_bt) * tiles + t if mode_name.endswith("cold") else blk // n_bt + t
            a0 = (first % n_at) * a_tile
            for i in range(AM):
                for j in range(4):
                    r = (i * 4 + j) & 15
                    m = (wave >> 1) * (32 * AM) + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)
                    n = (wave & 1) * 128 + j * 32 + (lane & 31)
                    exp[blk] += C[a0 + m, b0 + n]
    return exp


@pytest.mark.parametrize("mode_name", ["loop_kc_kr", "loop_kc_kc", "half_kc_kr", "loop_kc_kr_cold"])
@pytest.mark.parametrize("k,tiles", [(768, 3), (64, 1)])
def test_probe_loops_accumulate_the_right_products(mode_name, k, tiles):
    mode = B.PROBE_MODES.index(mode_name)
    a_rows, b_rows, wgs = 1024, 512, 6
    g = torch.Generator(device="cuda").manual_seed(5)
    A = torch.randn(a_rows, k, device="cuda", generator=g).to(torch.bfloat16)
    Bm = torch.randn(b_rows, k, device="cuda", generator=g).to(torch.bfloat16)
    BT = Bm.t().contiguous()
    sink = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
    print(f"[case] probe {mode_name} k={k} tiles={tiles}", flush=True)
    assert B.flce_probe(mode, A, Bm, BT, a_rows, b_rows, k, wgs, tiles, sink, torch.cuda.current_stream()) == B.FLCE_OK
    torch.cuda.synchronize()
    C = (A.double().cpu() @ Bm.double().cpu().t()).numpy()
    exp = _expected(C, mode_name, wgs, tiles, a_rows, b_rows)
    got = sink.cpu().double().numpy().reshape(wgs, 256)
    # fp32 accumulation of bf16 products over K and the few additions of the sink: far inside 1e-4 of the scale
    assert np.abs(got - exp).max() <= 1e-4 * np.abs(exp).max()
