"""The entry point that allocates nothing (synk_sliced_eval_static: partial results in a fixed
array inside the library's device image) against the entry point it is a variant of
(synk_sliced_eval with a caller's workspace), through the C ABI: two calls in a row, the second on
a smaller input, every output bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def synk():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1710_04162_amd import binding
    return binding


def _outputs(rows, classes):
    z = lambda n, dt, fill: torch.full((n,), fill, dtype=dt, device="cuda")
    return (z(1, torch.float32, -7.0), z(classes, torch.int32, -1), z(1, torch.float32, -7.0),
            z(1, torch.float32, -7.0), z(1, torch.int32, -1), z(rows, torch.int32, -1))


def _both(synk, rows, classes, n_slices, seed):
    rng = np.random.default_rng(seed)
    logits = torch.from_numpy((rng.standard_normal((rows, classes)) * 2.0).astype(np.float32)).cuda()
    labels = torch.from_numpy(rng.integers(0, classes, rows).astype(np.int32)).cuda()
    ws = torch.empty(synk.synk_sliced_eval_workspace_bytes(rows, classes, n_slices), dtype=torch.uint8, device="cuda")
    want, got = _outputs(rows, classes), _outputs(rows, classes)
    synk.synk_sliced_eval(logits, labels, n_slices, *want, ws)
    before = torch.cuda.memory_allocated()
    synk.synk_sliced_eval_static(logits, labels, n_slices, *got)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    names = ("ce_sum", "class_counts", "max_logit", "min_logit", "n_correct", "argmax")
    for name, a, b in zip(names, got, want):
        assert torch.equal(a, b), (name, rows, classes, n_slices)
    # and against what the outputs mean
    am = torch.argmax(logits, dim=1).to(torch.int32)
    assert torch.equal(got[5], am) and int(got[1].sum()) == rows
    assert int(got[4][0]) == int((am == labels).sum())


def test_static_scratch_entry_point_matches_workspace_entry_point(synk):
    synk.synk_static_scratch_init()
    _both(synk, 4096, 1000, 64, 1)      # the regular kernel: 8 chunks a slice
    _both(synk, 1000, 1000, 7, 2)       # smaller, ragged slices: the array still holds the first call's partials
    _both(synk, 130, 37, 3, 3)          # scalar path
    _both(synk, 4096, 1000, 64, 1)      # the first case again after the smaller ones


def test_static_scratch_limit_is_an_error_not_a_launch(synk):
    rows, classes, n_slices = 8 * 70000, 4, 1           # 70,000 chunks of partials: beyond the fixed array
    assert synk.synk_sliced_eval_workspace_bytes(rows, classes, n_slices) > (1 << 20)
    logits = torch.zeros((rows, classes), device="cuda")
    labels = torch.zeros(rows, dtype=torch.int32, device="cuda")
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_eval_static(logits, labels, n_slices, *_outputs(rows, classes))
    assert e.value.status == -6
