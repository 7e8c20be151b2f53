"""forest_predict_static -- the entry point for callers that cannot allocate -- against
forest_predict, through the C ABI: same bits, on two calls in a row (the second with a smaller
input, so that whatever the first left in the static scratch array is still there), for every
kernel family; sizes beyond the array are refused, large batches (no workspace) always run."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _models():
    yield "rank, full trees", wl.make_workload("c2", n_rows=1, n_trees=120).forest
    yield "rank, 10 classes", wl.make_workload("c4", n_rows=1, n_trees=200).forest
    yield "LDS rank, irregular", wl.make_workload("c5", n_rows=1, n_trees=40).forest
    yield "plain LDS, 300 features", wl.random_forest(902, n_trees=96, n_features=300, max_depth=7, stop_prob=0.1,
                                                    n_outputs=20, leaf_width=20, transform=wl.TRANSFORM_SOFTMAX,
                                                    aggregate=wl.AGG_MEAN)


@pytest.mark.parametrize("what,forest", list(_models()), ids=lambda v: v if isinstance(v, str) else "")
def test_static_entry_point_matches_forest_predict(what, forest):
    import torch
    import paper_2301_13441_amd as pk
    f = pk.forest_load(forest)
    try:
        rng = np.random.default_rng(len(what))
        for rows in (2500, 700, 1, 100000):       # smaller second call; one row; a batch that needs no workspace
            X = torch.from_numpy(rng.standard_normal((rows, forest.n_features)).astype(np.float32)).cuda()
            nbytes = max(f.out_bytes(rows), 4)
            want = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            got = torch.full((nbytes,), 0xAB, dtype=torch.uint8, device="cuda")
            f.predict(X, out=want)
            torch.cuda.synchronize()
            f.predict(X, out=got, static=True)
            torch.cuda.synchronize()
            assert torch.equal(got[:f.out_bytes(rows)], want[:f.out_bytes(rows)]), (what, rows)
    finally:
        f.close()


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2301_13441_amd as pk
    from paper_2301_13441_amd.binding import ForestError
    w = wl.make_workload("c5", n_rows=1, n_trees=128)      # 256 rank registers: 64 KB of ranks per 128 rows
    f = pk.forest_load(w.forest)
    try:
        assert f.info["kernel_path"] == 3
        rows = 40000                                        # 313 tiles x 64 KB > 8 MiB, and still a small batch
        assert rows < f.info["small_batch_rows"]
        X = torch.zeros((rows, 256), dtype=torch.float32, device="cuda")
        out = torch.zeros(max(f.out_bytes(rows), 4), dtype=torch.uint8, device="cuda")
        with pytest.raises(ForestError) as err:
            f.predict(X, out=out, static=True)
        assert err.value.code == -7                         # FOREST_ELIMIT
        f.predict(X, out=out)                               # the handle's own workspace takes it
        torch.cuda.synchronize()
    finally:
        f.close()
