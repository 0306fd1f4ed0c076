"""Full-size parity: every fwd+bwd workload bench.py can time (the three of the workload list and the
three shape variants: 32 and 128 slots, the paper's own five-head 2.7B shape), in the launch
configuration it times, every sequence and head compared element by element against the fp64 oracle
(the oracle finishes each of them in seconds on the host cores)."""
import pytest

from tests.test_gpu_bwd import compare_bwd, run_fwd_bwd

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["layer_1p3b", "layer_2p7b", "packed_16k", "layer_1p3b_m32", "layer_1p3b_m128",
                                  "layer_2p7b_h5"])
def test_full_size_fwd_bwd(oracle, name):
    from paper_2409_07146_amd import synth
    cfg = synth.CONFIGS[name] if name in synth.CONFIGS else synth.VARIANTS[name]
    x, got = run_fwd_bwd(cfg)
    rep = []
    try:
        compare_bwd(oracle, cfg, x, got, report=rep)
    finally:
        worst = {}
        for n, r, a, _ in rep:
            key = n.split("[")[0]
            w = worst.get(key, (0.0, 0.0))
            worst[key] = (max(w[0], r), max(w[1], a))
        print("\n%s worst (rel-L2, max-abs) per tensor: %s" % (
            name, {k: ("%.2e" % v[0], "%.2e" % v[1]) for k, v in worst.items()}))
