"""The diagnostic probe kernel runs in every mode and leaves finite values (its timings are read by
`bench.py --issue-overlap-probe`, not judged here)."""
import pytest

pytestmark = pytest.mark.gpu


def test_probe_runs_in_every_mode():
    import torch
    from paper_1907_03329_amd import binding
    out = torch.full((2 * 256 * 256,), float("nan"), dtype=torch.float32, device="cuda")
    for per_cu in (1, 2):
        for mode in (0, 1, 2, 3):
            if mode == 3 and per_cu == 1:
                with pytest.raises(binding.EsrnnError):
                    binding.esrnn_probe_issue_overlap(mode, 8, per_cu, out)
                continue
            out.fill_(float("nan"))
            binding.esrnn_probe_issue_overlap(mode, 8, per_cu, out)
            torch.cuda.synchronize()
            n = 256 * per_cu * 256
            assert torch.isfinite(out[:n]).all()
            assert torch.isnan(out[n:]).all()
    with pytest.raises(ValueError):
        binding.esrnn_probe_issue_overlap(0, 8, 2, out[:1000])
