"""mesa_mfma_probe (a measurement helper): the flop count the benchmark divides by is honest only if the kernel really
multiplies the operands it says it does -- the sum over a wave's 128 x 128 tile is recomputed here from the operand
pattern (sum over k of the column sums of A times the column sums of B), for operands kept in registers and for
operands read from LDS step by step."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def M():
    import paper_2111_11124_amd as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def pattern_words(idx):
    """the probe's operand pattern: word number -> two binary16 values of magnitude 1/2 .. 1"""
    x = idx.astype(np.uint64)
    mask = np.uint64(0xFFFFFFFF)
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & mask
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & mask
    x ^= x >> np.uint64(16)
    return ((x & np.uint64(0x83FF83FF)) | np.uint64(0x38003800)).astype(np.uint32)


def wave_tile_sum(block, wave, steps, from_lds):
    vec0 = block * 4096 + wave * 1024
    total = 0.0
    for s in range(steps):
        base = (s * 8) if from_lds else 0
        sums = []
        for side in (0, 4):                                  # A fragments 0..3, B fragments 4..7
            k_sums = np.zeros(16, np.float64)
            for f in range(4):
                v = vec0 + ((base + side + f) * 64 + np.arange(64)) % 1024      # the lanes' vectors
                words = pattern_words((v[:, None] * 4 + np.arange(4)[None, :]).reshape(-1))
                halves = words.view(np.float16).astype(np.float64).reshape(64, 8)   # lane l: row l%32, k = 8*(l/32) + e
                k_sums[0:8] += halves[:32].sum(axis=0)
                k_sums[8:16] += halves[32:].sum(axis=0)
            sums.append(k_sums)
        total += float(np.dot(sums[0], sums[1]))
    return total


@pytest.mark.parametrize("form,steps", [(0, 1), (0, 3), (1, 1), (1, 4)])
def test_probe_multiplies_what_it_says(M, form, steps):
    sink = torch.full((65536,), float("nan"), device="cuda")
    M.mesa_mfma_probe(form, steps, None, sink)
    torch.cuda.synchronize()
    got = sink.double().cpu().numpy().reshape(256, 4, 64).sum(axis=2)
    for block, wave in [(0, 0), (0, 3), (17, 1), (255, 2)]:
        ref = wave_tile_sum(block, wave, steps, form == 1)
        scale = 128 * 128 * 16 * steps * 0.6                 # sum of |products|, roughly
        assert abs(got[block, wave] - ref) <= 1e-5 * scale, (block, wave, got[block, wave], ref)


def test_probe_with_tile_loads_and_edge_cases(M):
    sink = torch.full((65536,), float("nan"), device="cuda")
    M.mesa_mfma_probe(1, 0, None, sink)
    torch.cuda.synchronize()
    assert float(sink.abs().max()) == 0.0
    gen = torch.Generator(device="cuda").manual_seed(3)
    feed = torch.randn(1 << 20, device="cuda", generator=gen).half()        # 2 MiB
    for form in (2, 3):
        out = []
        for _ in range(2):
            sink.fill_(float("nan"))
            M.mesa_mfma_probe(form, 37, feed, sink)
            torch.cuda.synchronize()
            out.append(sink.clone())
        assert bool(torch.isfinite(out[0]).all()) and torch.equal(out[0], out[1])
    with pytest.raises(M.MesaError):
        M.mesa_mfma_probe(2, 5, feed[:1000], sink)            # feed below 2 MiB
    with pytest.raises(M.MesaError):
        M.mesa_mfma_probe(4, 5, None, sink)
