"""GPU parity at the baseline's full shapes, in the launch configuration bench.py times: the
oracle runs whole micro-batches at full size (tens of seconds of fp64 numpy per case), so every
output element and every gradient is compared, not a sample."""
import numpy as np
import pytest

import synth_inputs as si
from tests import harness as hz
from tests.test_gpu_schedule import _run_iteration

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def _report(tag, errs):
    worst = sorted(errs.items(), key=lambda kv: -kv[1])[:3]
    print(tag, "worst:", [(k, f"{v:.2e}") for k, v in worst], flush=True)


def test_cfg1_gpt_h2048_two_microbatches():
    """4 layers, H 2048, 16 heads, S 2048, B 1, causal: forward, backward and the fp32
    accumulation of two micro-batches against the oracle's sum."""
    errs = hz.run_fwd_bwd_parity(si.CONFIGS[1], n_micro=2)
    _report("cfg1", errs)


def test_cfg2_bert_h1024_padded():
    """6 layers, H 1024, 16 heads (d 64), S 512, B 8, key padding 256..512."""
    errs = hz.run_fwd_bwd_parity(si.CONFIGS[2], n_micro=1)
    _report("cfg2", errs)


def test_cfg3_gpt_h5120_one_layer():
    """H 5120, 40 heads, MLP 20480, S 2048, B 2 at full width; one of the config's two layers
    (the second layer repeats the same kernels on the same shapes)."""
    cfg = si.scaled(si.CONFIGS[3], name="cfg3_one_layer", layers=1)
    errs = hz.run_fwd_bwd_parity(cfg, n_micro=1)
    _report("cfg3", errs)


def test_cfg4_v_schedule_full():
    """The single-GPU BitPipe iteration: 16 layers as 8 stages x 2 layers, D = 4, 8 micro-batches,
    H 1024, S 1024: loss and every accumulated gradient against the non-pipelined full-batch oracle."""
    loss, grads, worst = _run_iteration(si.CONFIGS[4], 4)
    print("cfg4 loss", loss, "worst grad err", f"{worst:.2e}", flush=True)


def test_cfg5_bert64_stage_d40_two_layers():
    """One stage of the paper's BERT-64 (Table 3) at its own width: H 2560, 64 heads of width 40
    (padded to 64 inside the attention kernels), S 512, B 4, key padding; two of the stage's
    four layers (the others repeat the same kernels on the same shapes)."""
    cfg = si.scaled(si.CONFIGS[5], name="cfg5_two_layers", layers=2)
    errs = hz.run_fwd_bwd_parity(cfg, n_micro=1)
    _report("cfg5", errs)


def test_cfg6_gpt96_stage_d96_two_layers():
    """One stage of the paper's GPT-96 (Table 3): H 3072, 32 heads of width 96 (padded to 128),
    S 1024, B 1, causal; two of its six layers."""
    cfg = si.scaled(si.CONFIGS[6], name="cfg6_two_layers", layers=2)
    errs = hz.run_fwd_bwd_parity(cfg, n_micro=2)
    _report("cfg6", errs)
