"""The streaming-bandwidth probe of the boundary: argument checking, and rates of a plausible size for the three
read/write mixes (a plain copy cannot beat a plain read)."""
import pytest

pytestmark = pytest.mark.gpu


def test_probe_rates_and_argument_errors():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2602_11470_amd import binding as B
    read = B.hbm_probe(B.CM_PROBE_READ, 1 << 30, 3)
    copy = B.hbm_probe(B.CM_PROBE_COPY, 1 << 30, 3)
    mix = B.hbm_probe(B.CM_PROBE_READ3_WRITE1, 1 << 30, 3)
    assert 500.0 < copy < read < 8000.0 and 500.0 < mix < 8000.0, (read, copy, mix)
    for bad in [(7, 1 << 30, 3), (B.CM_PROBE_READ, 1 << 20, 3), (B.CM_PROBE_READ, 1 << 30, 0)]:
        with pytest.raises(B.CachemirError) as e:
            B.hbm_probe(*bad)
        assert e.value.status == -1
