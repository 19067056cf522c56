"""GPU parity of the stage forward/backward against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

import synth_inputs as si
from tests import harness as hz

pytestmark = pytest.mark.gpu


def test_cfg0_tiny_gpt_fp32_full():
    """Tiny GPT-style stage in fp32: all 4 micro-batches, gradients accumulated; bound 1e-4."""
    errs = hz.run_fwd_bwd_parity(si.CONFIGS[0])
    print({k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("name,kw", [
    ("gpt_d64", dict(layers=2, hidden=256, heads=4, seq=192, microbatch=2, causal=True)),
    ("gpt_d128_ragged", dict(layers=2, hidden=256, heads=2, seq=200, microbatch=1, causal=True)),
    ("bert_d64_padded", dict(layers=2, hidden=256, heads=4, seq=160, microbatch=3, causal=False,
                             len_lo=40, len_hi=160)),
    ("bert_full_len", dict(layers=1, hidden=128, heads=2, seq=96, microbatch=2, causal=False)),
])
def test_small_bf16_stages(name, kw):
    cfg = si.scaled(si.CONFIGS[1], name="small_" + name, n_micro=2, **kw)
    errs = hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1)
    worst = max(errs.items(), key=lambda kv: kv[1])
    print(name, "worst", worst)


def test_small_fp32_bert_padded():
    cfg = si.scaled(si.CONFIGS[0], name="small_f32_bert", causal=False, len_lo=10, len_hi=64,
                    microbatch=3, n_micro=2)
    hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1)


def test_state_errors():
    import paper_2410_19367_amd as bp
    cfg = si.scaled(si.CONFIGS[0], name="state", layers=1)
    with hz.GpuStage(cfg, max_inflight=2) as g:
        x = hz.to_dev(si.make_activation(cfg, "act_in", 0), cfg.dtype)
        out = hz.empty_like_dev(tuple(x.shape), cfg.dtype)
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_backward(g.h, 0, 0, x, out)
        assert e.value.code == bp.BP_ESTATE
        bp.bp_stage_forward(g.h, 0, 0, x, out)
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_forward(g.h, 0, 0, x, out)
        assert e.value.code == bp.BP_ESTATE
        bp.bp_stage_forward(g.h, 0, 1, x, out)
        with pytest.raises(bp.BitPipeError) as e:      # max_inflight = 2
            bp.bp_stage_forward(g.h, 0, 2, x, out)
        assert e.value.code == bp.BP_ESTATE
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_forward(g.h, 1, 0, x, out)
        assert e.value.code == bp.BP_EINVAL
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_set_seqlens(g.h, 0, np.array([3, 3], dtype=np.int32))
        assert e.value.code == bp.BP_ESTATE       # causal stage
        bp.bp_stage_backward(g.h, 0, 1, x, out)
        bp.bp_stage_backward(g.h, 0, 0, x, out)
        with pytest.raises(bp.BitPipeError):
            bp.bp_stage_set_param(g.h, 0, 0, bp.TENSOR_IDS["wo"], np.zeros(7, dtype=np.float32))
    with pytest.raises(bp.BitPipeError) as e:
        bp.bp_stage_init(1, 100, 3, 8, 1, 1)
    assert e.value.code == bp.BP_ESHAPE
