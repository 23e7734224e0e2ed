"""Host-side checks of the shape-search tool (no GPU work)."""
import pytest


def test_tune_lists_only_shapes_the_library_accepts():
    ks = pytest.importorskip("paper_2603_18695_amd")
    from paper_2603_18695_amd import tune
    for waves in tune.WAVES:
        ks.ks_set_option("waves", waves)
        for form in tune.FORMS[waves]:
            ks.ks_set_option("form", form)
    for rows in tune.ROWS:
        ks.ks_set_option("rows", rows)
    for name, v in (("waves", 0), ("rows", 0), ("form", -1)):
        ks.ks_set_option(name, v)


def test_tune_refuses_to_run_without_a_gpu_or_for_unknown_pairs(capsys):
    import torch
    from paper_2603_18695_amd import tune
    if torch.cuda.is_available():
        assert tune.main(["--dtype", "affine_f32", "--op", "sum"]) == 2
    else:
        assert tune.main(["--dtype", "f32", "--op", "sum"]) == 2
    assert capsys.readouterr().err
