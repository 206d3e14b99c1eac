"""Non-uniform per-layer budgets: every layer has its own sketch width, Recent
and Candidate sizes (kvr_synth.layer_budgets); each layer's decode steps must
follow the oracle exactly as with a uniform budget."""
import pytest

import kvr_synth as S
from tests.test_gpu_parity import run_decode_steps, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kvr():
    from paper_2512_17917_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def LayerState():
    from paper_2512_17917_amd.state import LayerState as LS
    return LS


def test_layers_with_different_budgets_follow_the_oracle(kvr, LayerState):
    base = S.small_workload("lb", layers=3, batch=1, n_q_heads=8, n_kv_heads=2, context=800, budget=0.25, r=3,
                            steps=3, cfg_id=92)
    per_layer = S.layer_budgets(base, [0.5, 1.0, 1.5])
    sizes = [(w.w, w.n_recent, w.n_candidate) for w in per_layer]
    say("layer budgets", sizes)
    assert len(set(sizes)) == 3
    for layer, wl in enumerate(per_layer):
        run_decode_steps(kvr, LayerState, wl, layer, 2, fused=True)
