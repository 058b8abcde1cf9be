"""The GEMM kernels evaluate their work list with wave-parallel code (prefix sums and ballots over
the experts) when a shard has more than a handful of experts; the plain loops in the same library,
which the CPU tests check against the definition, are the reference.  Both must agree on every workgroup of every routing: bit-exact integer work."""
import numpy as np
import pytest
import torch

from paper_2508_19373_amd import binding as B

pytestmark = pytest.mark.gpu


def _routings(rng, n_local, max_rows):
    yield np.zeros(n_local, dtype=np.int64)
    yield np.full(n_local, 256, dtype=np.int64)
    for trial in range(12):
        R = int(rng.integers(0, max_rows + 1))
        cuts = np.sort(rng.integers(0, R + 1, size=n_local - 1))
        counts = np.diff(np.concatenate([[0], cuts, [R]]))
        if trial % 4 == 1:
            counts = (counts // 256) * 256
        if trial % 4 == 2:
            counts[rng.integers(0, n_local, size=max(1, n_local // 2))] = 0   # many empty experts
        if trial % 4 == 3:   # sizes around the class boundaries
            counts = rng.choice([1, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 385, 449, 512], n_local)
        yield counts.astype(np.int64)


@pytest.mark.parametrize("n_local,ncb,nk,max_slices,max_rows", [
    (8, 112, 64, 0, 9000),        # Mixtral GEMM1
    (8, 16, 224, 16, 9000),       # Mixtral GEMM2
    (2, 16, 224, 16, 3000),       # expert-parallel shard, small launches
    (2, 16, 224, 16, 20000),
    (1, 14, 320, 16, 5000),       # one shared expert
    (60, 11, 32, 0, 17000),       # Qwen1.5-MoE GEMM1
    (60, 8, 22, 2, 17000),
    (64, 14, 40, 5, 33000),       # Qwen2-57B-A14B GEMM2
    (65, 3, 40, 5, 9000),         # more experts than lanes
    (200, 2, 64, 8, 30000),
    (256, 1, 128, 16, 40000),     # the most experts the library takes
    (256, 5, 16, 0, 40000),
    (3, 1, 16, 2, 900),
    (4, 16, 224, 16, 6000),       # the last count the kernels walk with plain loops ...
    (5, 16, 224, 16, 6000),       # ... and the first they take wave-parallel
    (4, 28, 64, 0, 6000),
    (5, 28, 64, 0, 6000),
])
def test_wave_parallel_work_list_equals_the_plain_one(n_local, ncb, nk, max_slices, max_rows):
    rng = np.random.default_rng(n_local * 7919 + ncb)
    for counts in _routings(rng, n_local, max_rows):
        offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        cap = max(int(offs[-1]), 1) + int(rng.integers(0, 700))
        dev = B.moe_debug_device_units(torch.from_numpy(offs).cuda(), cap, ncb, nk, max_slices)
        torch.cuda.synchronize()
        dev = dev.cpu().numpy()
        if max_slices == 0:
            host = B.moe_debug_gemm_units(offs, cap, ncb)
            assert dev.shape[0] == host.shape[0]
            assert np.array_equal(dev[:, :5], host), counts
            live = dev[:, 0] > 0
            assert (dev[live, 5] == 0).all() and (dev[live, 6] == 0).all() and (dev[live, 7] == nk).all()
        else:
            # a shard whose down projection has this many column blocks and k-tiles
            shard = B.make_shard(n_local, n_local, 0, 256 * ncb, 64 * nk, 64 * nk)
            info, host = B.moe_debug_down_slices(offs, cap, shard, with_units=True)
            assert max_slices == min(16, nk // 8)     # what the library launches for this K
            assert dev.shape[0] == host.shape[0]
            assert np.array_equal(dev[:, [0, 1, 2, 4, 5, 6, 7]], host[:, :7]), counts
            live = dev[:, 0] > 0
            assert np.array_equal(dev[live, 8], host[live, 7]), counts
            ends = offs[dev[live, 1] + 1]
            assert np.array_equal(dev[live, 3], ends)


@pytest.mark.parametrize("n_local,ncb,max_rows", [(60, 11, 17000), (64, 14, 20000), (4, 8, 2000), (5, 8, 2000),
                                                  (200, 2, 60000), (1, 3, 700)])
def test_even_work_list_on_the_device_equals_the_host_one(n_local, ncb, max_rows):
    rng = np.random.default_rng(n_local * 31 + ncb)
    for counts in _routings(rng, n_local, max_rows):
        offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        cap = max(int(offs[-1]), 1) + int(rng.integers(0, 700))
        dev = B.moe_debug_device_units(torch.from_numpy(offs).cuda(), cap, ncb, 32, -1)
        torch.cuda.synchronize()
        dev = dev.cpu().numpy()
        host = B.moe_debug_even_units(offs, cap, ncb)
        assert dev.shape[0] == host.shape[0]
        assert np.array_equal(dev[:, :5], host), counts
