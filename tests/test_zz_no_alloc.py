"""The entry point that allocates nothing (tsr_project_core_static) against tsr_project_core:
same kernels on the library's built-in scratch, so the cores must be bit-identical; two calls in
a row on the shared scratch, the second with a smaller input."""
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tsr():
    import paper_2602_08007_amd as t
    assert torch.cuda.is_available()
    return t


def _case(tsr, m, n, r, dtype, precision, key):
    sig = si.make_signal(m, n, min(r, 16), "1/i", si.stream_key(key, 0))
    G = si.gradient(sig, 1e-3, si.stream_key(key, 1), dtype=dtype).to("cuda")
    U = si.orthonormal(m, r, si.stream_key(key, 2)).float().to("cuda")
    V = si.orthonormal(n, r, si.stream_key(key, 3)).float().to("cuda")
    C_ref = torch.full((r, r), float("nan"), device="cuda")
    tsr.tsr_project_core(G, U, V, C_ref, precision=precision)
    return G, U, V, C_ref


@pytest.mark.parametrize("dtype,prec", [(torch.float32, "split"), (torch.bfloat16, "bf16")])
def test_static_scratch_project_matches_workspace_project(tsr, dtype, prec):
    precision = tsr.TSR_PREC_SPLIT if prec == "split" else tsr.TSR_PREC_BF16
    big = _case(tsr, 768, 2048, 256, dtype, precision, 9101)         # k-split partials: most of the scratch
    small = _case(tsr, 200, 333, 17, dtype, precision, 9102)         # ragged, a corner of the scratch
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    for (G, U, V, C_ref) in (big, small, big):
        r = U.shape[1]
        C = torch.full((r, r), float("nan"), device="cuda") if False else C_ref.clone().fill_(float("nan"))
        tsr.tsr_project_core_static(G, U, V, C, precision=precision)
        torch.cuda.synchronize()
        assert torch.equal(C, C_ref)
        # alpha / accumulate on the shared scratch: C <- C + 0.5 * core, as tsr_project_core does it
        C2 = C_ref.clone()
        tsr.tsr_project_core(G, U, V, C2, alpha=0.5, accumulate=True, precision=precision)
        tsr.tsr_project_core_static(G, U, V, C, alpha=0.5, accumulate=True, precision=precision)
        torch.cuda.synchronize()
        assert torch.equal(C, C2)
    # beyond the built-in scratch: refused with its own status, nothing launched
    m, n, r = 2048, 5464, 512
    assert tsr.tsr_project_workspace_bytes(m, n, r) > tsr.TSR_PROJECT_STATIC_SCRATCH_BYTES
    G = torch.zeros(m, n, device="cuda", dtype=dtype); U = torch.zeros(m, r, device="cuda"); V = torch.zeros(n, r, device="cuda")
    C = torch.zeros(r, r, device="cuda")
    with pytest.raises(tsr.TsrError) as e:
        tsr.tsr_project_core_static(G, U, V, C, precision=precision)
    assert e.value.status == -6
