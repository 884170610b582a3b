"""GPU FedAvg (SplitLoRA step b2, Eq. 8-9) and SGD step (Eq. 4-5): bit-exact against the fixed-order
fp32 references, close to the fp64 oracle."""
import numpy as np
import pytest

from oracle import cref
from oracle import slora_oracle as so
from paper_2407_00952_amd import binding as B
from paper_2407_00952_amd import synth
from gpu_util import say

pytestmark = pytest.mark.gpu


def _gpu_fedavg(vecs, counts, offset=0):
    import torch
    n = vecs[0].size
    dev = []
    for v in vecs:
        t = torch.empty(n + 4, dtype=torch.float32, device="cuda")
        t[offset:offset + n] = torch.from_numpy(v).cuda()
        dev.append(t[offset:offset + n])
    out = torch.full((n + 4,), float("nan"), dtype=torch.float32, device="cuda")
    B.slora_fedavg(dev, counts, n, out[offset:offset + n])
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    assert np.all(np.isnan(res[:offset])) and np.all(np.isnan(res[offset + n:]))
    return res[offset:offset + n]


@pytest.mark.parametrize("K,n,offset", [(16, None, 0), (1, 1000, 0), (3, 4099, 0), (5, 1023, 1), (64, 257, 0), (2, 3, 0)])
def test_fedavg_bit_exact(K, n, offset):
    """K = 16, n = None is workload 5's aggregation: 16 clients x 1 769 472 fp32 adapter parameters."""
    vecs, counts = synth.make_fedavg_inputs(n_clients=K, n_params=n)
    say("fedavg K=%d n=%d offset=%d" % (K, vecs[0].size, offset))
    got = _gpu_fedavg(vecs, counts, offset)
    ref = cref.fedavg_f32(vecs, counts)
    assert got.tobytes() == ref.tobytes()
    o64 = so.fedavg(vecs, counts)
    assert np.abs(got - o64).max() <= 1e-6 * np.abs(o64).max()


def test_fedavg_identities_on_gpu():
    vecs, counts = synth.make_fedavg_inputs(n_clients=4, n_params=5000)
    x = vecs[0]
    assert np.array_equal(_gpu_fedavg([x], [7]), x)
    assert np.array_equal(_gpu_fedavg([x] * 4, [9, 9, 9, 9]), x)
    assert np.array_equal(_gpu_fedavg(vecs, [3, 0, 0, 0]), x)
    with pytest.raises(B.SloraError) as e:
        _gpu_fedavg(vecs, [0, 0, 0, 0])
    assert e.value.code == B.SLORA_EZERO
