"""GPU parity at the full sizes of the 7B, 20B and 70B workloads, in the launch configuration
bench.py times (default tuning, verify on): fingerprints and plans of every
tensor against the oracle, every assembled slot against its host source, and
oracle-assembled samples byte for byte."""
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_harness import run_workload_both, say  # noqa: E402
from paper_2512_01357_amd import synth  # noqa: E402


def test_llama_7b_family_full_size():
    say("full size: llama 7B family")
    w = synth.workload_llama7b()
    plans, _ = run_workload_both(w)
    for v in ("v1", "v2", "v3"):
        p = plans[v]
        assert p.reused_bytes + p.transfer_bytes == w.models[v].nbytes
        assert 0.51 < p.reused_bytes / w.models[v].nbytes < 0.53


def test_neox_20b_fragmented_pool_full_size():
    say("full size: NeoX 20B into a fragmented 200 GB pool")
    w = synth.workload_neox20b()
    plans, before = run_workload_both(w)
    p = plans["M20"]
    assert before["n_free_regions"] >= 5
    assert p.reused_bytes + p.transfer_bytes == w.models["M20"].nbytes
    assert 0.29 < p.reused_bytes / w.models["M20"].nbytes < 0.32
    # the load used the holes, not only the tail of the pool
    assert min(op.dst_off for op in p.ops) < before["capacity"] - before["largest_free"]


def test_neox_20b_into_a_pool_that_is_too_small_full_size():
    say("full size: NeoX 20B, 72 GB pool with 59 GB retained: Stage 1 + Stage 2 + alias")
    w = synth.workload_neox20b_tight()
    plans, _ = run_workload_both(w)
    p = plans["M20"]
    assert len(p.evictions) > 1000 and p.evicted_bytes > 16e9
    # the bound is what lies inside the subspaces that take tensors: a fraction of the 59 GB resident
    assert p.moves and p.moved_bytes <= p.merge_bound < 10e9
    assert p.alias and 12.3e9 < p.reused_bytes < 12.5e9
    assert p.reused_bytes + p.transfer_bytes == w.models["M20"].nbytes


@pytest.mark.parametrize("reuse,overlap", [(0.0, False), (0.5, True), (0.9, False)])
def test_llama3_70b_full_size(reuse, overlap):
    """Config 5 as one model: one plan of 723 tensors (made without a host image), the missing
    tensors fed through a pinned segment smaller than the model (at 50 %: through its two
    halves, one refilled while the other is copied)."""
    say("full size: Llama-3 70B as one 723-tensor model, reuse %.0f %%%s"
        % (reuse * 100, ", cache halves refilled during the copies" if overlap else ""))
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    w = synth.workload_llama70b(reuse, int(free - (16 << 30)))
    plans, _ = run_workload_both(w, overlap=overlap)
    p = plans["M70"]
    total = w.models["M70"].nbytes
    assert len(p.ops) == 723 and p.reused_bytes + p.transfer_bytes == total
    assert abs(p.reused_bytes / total - reuse) < 0.02
    info = run_workload_both.last_infos["M70"]
    if reuse == 0.0:
        assert sum(1 for op in p.ops if op.kind == 0) == 0      # nothing resident, nothing reused
        assert info["feeds"] >= 3                               # 141 GB through a 48 GB segment
    if overlap:
        assert info["feeds"] >= 3                               # 70.6 GB through halves of 24 GB
    say("feeds: %d, library time %.3f s" % (info["feeds"], info["library_s"]))
