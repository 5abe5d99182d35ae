"""The streaming kernels without arithmetic (dvp_hbm_probe) that bench.py times next to the library's calls:
they must move what they say they move."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dvp():
    from paper_2512_23087_amd import dvp as binding
    binding.lib()
    return binding


@pytest.mark.parametrize("n,v", [(7, 4104), (300, 151936), (2, 8)])
def test_probe_modes_move_what_they_say(dvp, n, v):
    g = torch.Generator(device="cpu").manual_seed(n * 1000 + v)
    a = torch.randn(n, v, generator=g).to(torch.bfloat16).cuda()
    b = torch.randn(n, v, generator=g).to(torch.bfloat16).cuda()
    a0, b0 = a.clone(), b.clone()
    for mode in (dvp.PROBE_FILL, dvp.PROBE_FILL_WIDE):
        c = torch.full((n, v), 3.0, dtype=torch.bfloat16, device="cuda")
        dvp.hbm_probe(mode, a, b, c)
        torch.cuda.synchronize()
        assert torch.count_nonzero(c).item() == 0
    c = torch.full((n, v), 3.0, dtype=torch.bfloat16, device="cuda")
    dvp.hbm_probe(dvp.PROBE_ROWS_2R1W, a, b, c)
    torch.cuda.synchronize()
    assert torch.equal(c.view(torch.int16), a.view(torch.int16))      # a's rows out to c, bit for bit
    for mode in (dvp.PROBE_READ, dvp.PROBE_READ_ONESHOT):
        dvp.hbm_probe(mode, a, b, c)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), a0.view(torch.int16)) and torch.equal(b.view(torch.int16), b0.view(torch.int16))
    assert torch.equal(c.view(torch.int16), a.view(torch.int16))      # the reading modes write nothing


def test_probe_refuses_what_it_cannot_run(dvp):
    a = torch.zeros(4, 20 * 16384 // 2 + 8, dtype=torch.bfloat16, device="cuda")     # rows longer than 19 register slots
    with pytest.raises(dvp.DvpError) as e:
        dvp.hbm_probe(dvp.PROBE_ROWS_2R1W, a, a.clone(), a.clone())
    assert e.value.status == 5                                                        # DVP_ERR_UNSUPPORTED
    dvp.hbm_probe(dvp.PROBE_FILL, None, None, a)                                       # a fill needs no inputs
    torch.cuda.synchronize()
