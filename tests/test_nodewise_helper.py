"""The sampled node-wise evaluation helper used by the full-size GPU tests agrees with full layer-wise
oracle inference on a small graph (CPU)."""
import numpy as np
import torch

from dgi_inputs import configs
from oracle import oracle
from tests.helpers import nodewise_oracle


def test_nodewise_helper_matches_full_inference():
    for k, scale in [(1, 0.3), (4, 0.00005), (3, 0.001)]:
        cfg = configs.make_config(k, scale=scale)
        layers = configs.to_numpy_layers(cfg["layers"])
        full = oracle.infer(cfg["indptr"].numpy(), cfg["indices"].numpy(), layers, cfg["x"].float().numpy())
        deg = torch.diff(cfg["indptr"].to(torch.int64))
        targets = [int(torch.argmax(deg)), 0, 5, cfg["num_nodes"] - 1, 5]
        got = nodewise_oracle(cfg["indptr"], cfg["indices"], cfg["x"], layers, targets, len(layers))
        np.testing.assert_array_equal(got, full[targets])
