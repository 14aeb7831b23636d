"""Host logic of bench.py that needs no GPU: the single-GPU contract of its command line, and the committed HBM-traffic
measurements it quotes in `roofline.traffic` against the bytes the kernels have to move by the size formulas
(Sec. 4.6: n*B*D/8 bytes of codes, plus the block scales; a step streams P twice and g, w once each)."""
import importlib.util
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.parametrize("gpus", [2, 8, 0])
def test_more_than_one_gpu_is_refused_with_a_message(gpus):
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", str(gpus), "--steps", "1", "--warmup", "0"],
                         capture_output=True, text=True, timeout=120)
    assert run.returncode != 0
    assert "single-GPU" in run.stderr and "--gpus 1" in run.stderr
    assert run.stdout.strip() == ""                       # no JSON line that could be mistaken for a measurement


def _p_bytes(D, n, bits, block, scale_bytes):
    ld = (D + 2047) // 2048 * 2048
    return n * ld * bits // 8 + n * (ld // block) * scale_bytes


def test_committed_traffic_figures_match_the_algorithmic_bytes():
    b = _bench()
    D, n = 25_557_032, 100
    cases = [("imagenet_resnet50_int8", _p_bytes(D, n, 8, 128, 4)), ("imagenet_resnet50_int4", _p_bytes(D, n, 4, 64, 2))]
    for tag, p in cases:
        proj = b.read_traffic(tag, "twa_project")
        expd = b.read_traffic(tag, "twa_expand_update")
        assert proj is not None and expd is not None, tag
        # projection: P and g read, n floats written; expansion: P and w read, w written
        assert abs(proj / (p + 4 * D + 4 * n) - 1) < 5e-3, (tag, proj)
        assert abs(expd / (p + 8 * D) - 1) < 5e-3, (tag, expd)
    # layer-wise (161 parameter tensors): the same streams; the 4-bit min-max codes carry no block scales
    for tag, p in (("layerwise_imagenet_resnet50_int8", _p_bytes(D, n, 8, 128, 4)), ("layerwise_imagenet_resnet50_minmax4", _p_bytes(D, n, 4, 64, 0))):
        proj = b.read_traffic(tag, "twa_beta_step")
        expd = b.read_traffic(tag, "twa_weights_from_beta")
        assert proj is not None and expd is not None, tag
        assert abs(proj / (p + 4 * D) - 1) < 5e-3, (tag, proj)          # (+1.3 % of tiles on layer boundaries read nothing twice)
        assert abs(expd / (p + 8 * D) - 1) < 5e-3, (tag, expd)
    # the batched projection of the fine-tuning shape: bf16 P read once, k = 8 gradients read
    Dv, nv, k = 86_567_656, 20, 8
    t = b.read_traffic("batched_vit_b16_finetune_bf16", "twa_project")
    assert t is not None
    assert abs(t / (2 * nv * ((Dv + 127) // 128 * 128) + 4 * k * Dv) - 1) < 5e-3, t


def test_no_traffic_figure_for_a_workload_nobody_measured():
    b = _bench()
    assert b.read_traffic("tiny_fp32", "twa_project") is None
    assert b.read_traffic("imagenet_resnet50_int8", "no_such_kernel") is None


def test_peaks_are_the_published_ones():
    b = _bench()
    assert b.HBM_PEAK_GBPS == 8000.0
    assert abs(b.VALU_PEAK_TLANE - 39.3216) < 1e-9       # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
