"""Deployment table of the library (paper Sec. 4.1) and the tools that fill it: host logic only,
no device call is made (attn_deploy_* and attn_deployed do not touch the GPU)."""
import json
import os

import pytest

import paper_2403_16863_amd as A
from paper_2403_16863_amd import deploy
from paper_2403_16863_amd import inputs as I


@pytest.fixture(autouse=True)
def clean_table():
    A.attn_deploy_clear()
    yield
    A.attn_deploy_clear()


def test_default_applies_until_something_is_deployed():
    for (N, d) in ((4096, 128), (100, 64), (4096, 64)):
        matched, v, h = A.attn_deployed(N, d, A.ATTN_BF16, True)
        assert not matched and h == -1 and v == A.attn_default_variant(N, d, A.ATTN_BF16, True)


def test_entries_match_by_shape_class_and_range_newest_first():
    A.attn_deploy_variant(10, 128, A.ATTN_BF16, True, 1024, 8192)
    assert A.attn_deployed(1024, 128, A.ATTN_BF16, True) == (True, 10, -1)
    assert A.attn_deployed(8192, 128, A.ATTN_BF16, True) == (True, 10, -1)
    for other in ((1023, 128, A.ATTN_BF16, True), (8193, 128, A.ATTN_BF16, True), (4096, 128, A.ATTN_BF16, False),
                  (4096, 128, A.ATTN_F16, True), (4096, 64, A.ATTN_BF16, True)):
        assert not A.attn_deployed(*other)[0]
    A.attn_deploy_variant(20, 128, A.ATTN_BF16, True, 4096, 4096)     # narrower and newer
    assert A.attn_deployed(4096, 128, A.ATTN_BF16, True) == (True, 20, -1)
    assert A.attn_deployed(4097, 128, A.ATTN_BF16, True) == (True, 10, -1)
    A.attn_deploy_clear()
    assert not A.attn_deployed(4096, 128, A.ATTN_BF16, True)[0]


def test_bad_requests_are_refused():
    nv = A.attn_num_variants()
    for args in ((nv, 128, A.ATTN_BF16, True, 1, 10), (-1, 128, A.ATTN_BF16, True, 1, 10), (0, 96, A.ATTN_BF16, True, 1, 10),
                 (0, 128, 7, True, 1, 10), (0, 128, A.ATTN_BF16, True, 0, 10), (0, 128, A.ATTN_BF16, True, 11, 10)):
        with pytest.raises(A.AttnError) as e:
            A.attn_deploy_variant(*args)
        assert e.value.code == -1
    d128_only = next(v for v in range(nv) if A.attn_variant_supported(v, 128, A.ATTN_BF16, True)
                     and not A.attn_variant_supported(v, 64, A.ATTN_BF16, True))
    with pytest.raises(A.AttnError) as e:                              # built, but not for this head dimension
        A.attn_deploy_variant(d128_only, 64, A.ATTN_BF16, True, 1, 10)
    assert e.value.code == -2
    for handle in (-1, 64, 63):                                        # out of range, and nothing loaded there
        with pytest.raises(A.AttnError):
            A.attn_deploy_codeobj(handle, 1, 10)
    with pytest.raises(A.AttnError):
        A.attn_deployed(0, 128, A.ATTN_BF16, True)
    assert not A.attn_deployed(4096, 128, A.ATTN_BF16, True)[0]        # nothing slipped in


def test_table_holds_sixteen_entries():
    for n in range(16):
        A.attn_deploy_variant(0, 128, A.ATTN_F16, False, 100 * n + 1, 100 * n + 100)
    with pytest.raises(A.AttnError) as e:
        A.attn_deploy_variant(0, 128, A.ATTN_F16, False, 5000, 6000)
    assert e.value.code == -2
    assert A.attn_deployed(1550, 128, A.ATTN_F16, False) == (True, 0, -1)
    A.attn_deploy_clear()
    A.attn_deploy_variant(0, 128, A.ATTN_F16, False, 5000, 6000)


def _ranking(tmp_path, name, label, best, gain, shape=None):
    body = {"workload": label, "best_variant": best, "best_vs_default": gain}
    if shape:
        body["shape"] = shape
    p = tmp_path / f"ranking_{name}.json"
    p.write_text(json.dumps(body))
    return str(p)


def test_a_ranking_is_deployed_only_for_a_gain_beyond_the_noise(tmp_path):
    label = "cfgx: B2 H32 N4096 d128 causal bf16"
    default = A.attn_default_variant(4096, 128, A.ATTN_BF16, True)
    other = 10 if default != 10 else 9
    assert deploy.deploy_ranking(_ranking(tmp_path, "a", label, default, 1.2)) is None    # best is the default
    assert deploy.deploy_ranking(_ranking(tmp_path, "b", label, other, 1.004)) is None    # inside the noise
    assert not A.attn_deployed(4096, 128, A.ATTN_BF16, True)[0]
    r = deploy.deploy_ranking(_ranking(tmp_path, "c", label, other, 1.05))
    assert r["variant"] == other and (r["n_min"], r["n_max"]) == (2049, 8191)
    assert A.attn_deployed(4096, 128, A.ATTN_BF16, True) == (True, other, -1)
    assert A.attn_deployed(2049, 128, A.ATTN_BF16, True)[0] and not A.attn_deployed(2048, 128, A.ATTN_BF16, True)[0]
    assert not A.attn_deployed(8192, 128, A.ATTN_BF16, True)[0]
    # the explicit shape entry wins over the label, and a directory is walked in file-name order
    A.attn_deploy_clear()
    _ranking(tmp_path, "d", "no shape in this label", 3 if A.attn_default_variant(512, 64, A.ATTN_F16, False) != 3 else 0, 1.1,
             {"B": 1, "H": 1, "N": 512, "d": 64, "causal": False, "dtype": I.F16})
    done = deploy.deploy_stored_rankings(str(tmp_path))
    assert [x["ranking"] for x in done] == ["ranking_c.json", "ranking_d.json"]
    assert A.attn_deployed(512, 64, A.ATTN_F16, False)[0] and A.attn_deployed(4096, 128, A.ATTN_BF16, True)[0]


def test_the_committed_rankings_parse_and_name_existing_variants():
    import glob
    paths = sorted(glob.glob(os.path.join(deploy.STORE_DIR, "ranking_*.json")))
    assert paths, "the package ships the rankings of its stored searches"
    for p in paths:
        s = json.load(open(p))
        shape = deploy.shape_of_ranking(s)
        assert shape["d"] in (64, 128) and shape["N"] >= 1
        assert 0 <= s["best_variant"] < A.attn_num_variants()
        assert A.attn_variant_supported(s["best_variant"], shape["d"], shape["dtype"], shape["causal"]) == 1
    # what ships today: no ranking beats the default by more than the noise, so nothing is deployed
    assert deploy.deploy_stored_rankings() == []
