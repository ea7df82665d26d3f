"""The entry point that allocates nothing (per_min_priority_static) against per_min_priority."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

from paper_2311_09445_amd import workloads as wl  # noqa: E402
from paper_2311_09445_amd.per import ERANGE, PerError, PrioritizedReplay  # noqa: E402


def fill(K, N, T, seed):
    rng = np.random.default_rng(seed)
    buf = PrioritizedReplay(K, N, T, ())
    prio = wl._draw_priorities("lognormal_0_1", rng, (T, N))
    prio[rng.random((T, N)) < 0.05] = 0.0
    buf.insert(N, None, torch.from_numpy(prio).cuda())
    return buf, prio, rng


def test_static_scratch_entry_point_equals_the_arena_one():
    print("per_min_priority_static: K=16 N=300001 T=3, then K=2 N=1000 T=1", flush=True)
    # first call: a large buffer (293 partial minima per tree in the static array)
    big, prio, rng = fill(16, 300001, 3, 1)
    out = torch.empty(3, dtype=torch.float32, device="cuda")
    big.min_priority_static(out)
    want = big.min_priority()
    torch.cuda.synchronize()
    assert out.cpu().numpy().tobytes() == want.cpu().numpy().tobytes()
    host = np.array([prio[t][prio[t] > 0].min() for t in range(3)], dtype=np.float32)
    assert out.cpu().numpy().tobytes() == host.tobytes()
    # second call in a row: a smaller input, which leaves most of what the first call wrote in the array
    small, prio2, _ = fill(2, 1000, 1, 2)
    out2 = torch.empty(1, dtype=torch.float32, device="cuda")
    small.min_priority_static(out2)
    want2 = small.min_priority()
    torch.cuda.synchronize()
    assert out2.cpu().numpy().tobytes() == want2.cpu().numpy().tobytes()
    assert out2.cpu().numpy()[0] == prio2[0][prio2[0] > 0].min()
    # and the large one again after an update that removes its minimum
    t0_min = int(np.argmin(np.where(prio[0] > 0, prio[0], np.inf)))
    big.update(torch.tensor([[t0_min], [0], [0]], dtype=torch.int32, device="cuda"),
               torch.tensor([[5.0], [prio[1][0]], [prio[2][0]]], dtype=torch.float32, device="cuda"))
    big.min_priority_static(out)
    assert out.cpu().numpy().tobytes() == big.min_priority().cpu().numpy().tobytes()
    # beyond the static array's size: refused with a clear error, nothing enqueued
    many = PrioritizedReplay(4, 64, 65, ())
    with pytest.raises(PerError) as err:
        many.min_priority_static()
    assert err.value.code == ERANGE
