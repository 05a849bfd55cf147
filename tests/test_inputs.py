"""The synthetic workload generator: shapes, determinism, statistics (CPU only)."""
import numpy as np
import torch

from oracle import rf2_oracle as orc
from paper_2512_24086_amd import inputs


def test_workload_table_matches_the_named_configs():
    w = inputs.WORKLOADS
    assert [w[k].N for k in ("tiny", "image", "video480p", "video720p", "longvideo")] == \
        [1536, 4096, 32760, 75600, 118800]
    assert w["video720p"].n_blocks == 591 and w["video720p"].heads == 40
    assert w["longvideo"].sweep == (0.5, 0.7, 0.8, 0.9) and w["longvideo"].sigma == 0.5


def test_generator_is_seeded_unit_variance_and_smooth():
    wl = inputs.WORKLOADS["tiny"]
    q, k, v = inputs.make_qkv(wl)
    assert q.shape == (1, 2, 1536, 64) and q.dtype == torch.bfloat16
    q2 = inputs.make_tensor(wl, 0)
    assert torch.equal(q, q2) and not torch.equal(q, k)
    only1 = inputs.make_tensor(wl, 0, heads=[1])
    assert torch.equal(only1[0, 0], q[0, 1])
    x = orc.bf16_bits_to_f64(inputs.bf16_bits(q))[0, 0]
    assert abs(x.std(axis=0).mean() - 1.0) < 0.02
    # neighbouring tokens along w are far more alike than distant ones
    g = x.reshape(6, 16, 16, 64)
    near = np.mean((g[:, :, 1:] - g[:, :, :-1]) ** 2)
    far = np.mean((g[:, :, 8:] - g[:, :, :-8]) ** 2)
    assert near < 0.5 * far


def test_bits_round_trip():
    t = torch.tensor([1.0, -2.5, 0.1], dtype=torch.bfloat16)
    assert orc.bf16_bits_to_f64(inputs.bf16_bits(t)).tolist() == t.double().tolist()
