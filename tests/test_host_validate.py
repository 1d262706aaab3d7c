"""bcp_validate_meta: the metadata checks of bcp_plan on the host (Sec. 3.2 records, Sec. 4.1 one saver
per shard), reachable without a GPU.  The GPU test test_gpu_parity.py::test_device_and_host_verdicts_agree
runs the same list through bcp_plan."""
import numpy as np
import pytest

from paper_2407_20143_amd import binding
from tests import meta_cases

CASES = meta_cases.cases()


@pytest.mark.parametrize("idx", range(len(CASES)), ids=[c[0] for c in CASES])
def test_status_per_case(idx):
    name, sm, tm, flags, want = CASES[idx]
    got, text = meta_cases.host_verdict(sm, tm, flags)
    assert got == want, f"{name}: {got} ({text})"


def test_the_message_names_the_record():
    _, sm, tm, _, _ = next(c for c in CASES if c[0] == "itemsize 3")
    _, text = meta_cases.host_verdict(sm, tm, 0)
    assert "saved record 0" in text
    _, sm, tm, _, _ = next(c for c in CASES if c[0] == "flat range beyond the box")
    _, text = meta_cases.host_verdict(sm, tm, 0)
    assert "target record 0" in text
    # the first bad record in (saved..., target...) order is the one reported
    _, sm, tm, _, _ = next(c for c in CASES if c[0] == "ok")
    sm = np.concatenate([sm, sm, sm])
    sm["byte_offset"] = [0, 128, 256]
    sm["itemsize"][1] = 5
    sm["ndim"][2] = 11
    assert meta_cases.host_verdict(sm, tm, 0)[0] == "BCP_ERR_INVALID_ARG"
    assert "saved record 1" in meta_cases.host_verdict(sm, tm, 0)[1]


def test_bad_arguments():
    L = binding.lib()
    assert L.bcp_status_name(L.bcp_validate_meta(None, 1, None, 0, 0)) == b"BCP_ERR_INVALID_ARG"
    assert L.bcp_status_name(L.bcp_validate_meta(None, 0, None, -1, 0)) == b"BCP_ERR_INVALID_ARG"
    assert L.bcp_status_name(L.bcp_validate_meta(None, 0, None, 0, 1 << 9)) == b"BCP_ERR_INVALID_ARG"
    assert L.bcp_status_name(L.bcp_validate_meta(None, 0, None, 0, binding.BCP_META_ON_DEVICE)) == b"BCP_ERR_INVALID_ARG"
    assert L.bcp_validate_meta(None, 0, None, 0, 0) == 0
