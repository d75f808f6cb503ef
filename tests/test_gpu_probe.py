"""The bandwidth probe that bench.py prints beside the roofline figure (a library of its own, include/cagra_probe.h):
it computes nothing of the method, so all there is to check is that both patterns run and that bad arguments are refused."""
import pytest

pytestmark = pytest.mark.gpu


def test_probe_patterns_run_and_bad_arguments_are_refused():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2308_15136_amd as cagra
    data = torch.zeros((4096, 128), dtype=torch.float32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    cagra.probe_bandwidth(data, pattern=0, sink=sink)
    for rif in (0, 2, 4, 8):
        for team in (0, 4, 8, 16, 32):
            cagra.probe_bandwidth(data, pattern=1, n_read=10_000, team_size=team, rows_in_flight=rif, sink=sink)
    torch.cuda.synchronize()
    for bad in (dict(pattern=2), dict(pattern=1, n_read=10, team_size=3), dict(pattern=1, n_read=10, rows_in_flight=5)):
        with pytest.raises(cagra.CagraError):
            cagra.probe_bandwidth(data, sink=sink, **bad)
    torch.cuda.synchronize()
