"""The comparison systems of the paper (Sec. 2.1, Sec. 2.2, Table 1) run through the same four calls: parity of the HIP
path with the oracle in each mode, on the small MLP workload's shape."""
import numpy as np
import pytest

from oracle import nets
from paper_2111_08274_amd import modes, synth
from tests.pair import Pair

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", modes.MODES)
def test_mode_parity_three_cycles(mode):
    cfg, x, y = synth.config_inputs(1, n_samples=128)
    fn, shape = nets.NETS["mlp"]
    a = modes.mode_arguments(mode, cfg["ratio"], cfg["n_select"], local_steps=3)
    p = Pair(fn(), shape, cfg["n_replicas"], a["n_select"], x, y, cfg["batch"], cfg["lr"], 0.9, a["ratio"],
             net_name="mlp", t_sync=a["t_sync"])
    want = modes.steps_per_cycle(mode, cfg["ratio"], local_steps=3)
    assert p.gpu.steps().tolist() == want.tolist() == p.cpu.steps.tolist()
    for cycle in range(3):
        p.local_steps()
        d_agg = p.select_aggregate(cycle)
        d = p.max_param_diff()
        print(mode, "cycle", cycle, "max |w_gpu - w_oracle|", d, "aggregate", d_agg, flush=True)
        assert d <= 1e-4 and d_agg <= 1e-4
    if mode != "hadfl":                       # every device is averaged: all flags set, equal weights
        sel, flag, w = p.gpu.selected()
        assert flag.all() and np.allclose(w, 1.0 / cfg["n_replicas"])
    p.close()
