"""The stream probes (measurement kernels, not part of the stage) leave the
arrays as they were in the read and in-place mixes, and copy in the copy mix."""
import pytest
import torch

from paper_2009_03816_amd import probes

pytestmark = pytest.mark.gpu


def arrays(K, D, ld):
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(5)
    return [torch.empty(K, ld, dtype=torch.float32, device="cuda:0").normal_(0.0, 1.0, generator=gen)
            for _ in range(3)]


@pytest.mark.parametrize("K,D,ld", [(3, 70_000, 70_000), (5, 4_100, 4_104)])
def test_stream_probe_mixes(K, D, ld):
    print(f"[case] stream probes K={K} D={D} ld={ld}", flush=True)
    x, v, p = arrays(K, D, ld)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    keep = [t.clone() for t in (x, v, p)]
    for mix in ("read", "inplace"):
        for chunked in (True, False):
            probes.pso_ps_probe_stream(mix, x, v, p, sink, K, D, ld, block_threads=64,
                                       chunked=chunked, super_tiles=8, chunk_tiles=2, wgs_per_cu=20)
    torch.cuda.synchronize()
    for t, k in zip((x, v, p), keep):
        assert torch.equal(t, k)
    probes.pso_ps_probe_stream("copy", x, v, p, sink, K, D, ld, block_threads=128, wgs_per_cu=64)
    torch.cuda.synchronize()
    # whole 16-byte groups of every row are copied; the ragged ends are skipped
    assert torch.equal(v[:, 4:D - 4], x[:, 4:D - 4]) and torch.equal(x, keep[0])
    assert float(sink.item()) == 0.0


def test_policy_probe_keeps_the_arrays():
    K, D, ld = 4, 33_000, 33_000
    print(f"[case] cache-policy probe K={K} D={D}", flush=True)
    x, v, p = arrays(K, D, ld)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    keep = [t.clone() for t in (x, v, p)]
    for loads in ("none", "nt", "sc0+nt", "nt+sc1", "sc0+nt+sc1"):
        for stores in ("none", "sc0", "nt", "sc1", "sc0+sc1", "nt+sc1"):
            probes.pso_ps_probe_policy(x, v, p, sink, K, D, ld, super_tiles=8, chunk_tiles=2,
                                       load_policy=probes.policy_bits(loads),
                                       store_policy=probes.policy_bits(stores))
    torch.cuda.synchronize()
    for t, k in zip((x, v, p), keep):
        assert torch.equal(t, k)
    with pytest.raises(RuntimeError):
        probes.pso_ps_probe_policy(x, v, p, sink, K, D, ld, load_policy=4)
