"""The C-ABI library loads without a GPU, exports every function that
include/ann.h declares, and rejects bad arguments on the host."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    text = (ROOT / "include" / "ann.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ann_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported():
    import paper_2503_17911_amd as ann
    names = declared_functions()
    assert len(names) >= 10
    lib = ctypes.CDLL(str(ann.LIB_PATH))
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in ann.h but not exported"
    assert sorted(ann.EXPORTED_SYMBOLS) == names
    for name in names:
        assert hasattr(ann, name), f"binding lacks {name}"


def test_host_side_argument_checks():
    import paper_2503_17911_amd as ann
    with pytest.raises(ann.AnnError) as e:
        ann.ann_upload_index(n=0, d=4, degree=2, metric=0, vectors=None, levels=[(8, None, None, None, None)],
                             adjacency=None, entry_point=0)
    assert e.value.status == ann.EINVAL
    with pytest.raises(ann.AnnError) as e:
        ann.ann_upload_index(n=10, d=4, degree=200, metric=0, vectors=None, levels=[(8, 1, 1, 1, 1)], adjacency=1,
                             entry_point=0)
    assert e.value.status == ann.ECAPACITY
    with pytest.raises(ann.AnnError) as e:
        ann.ann_upload_index(n=10, d=5, degree=2, metric=0, vectors=None, levels=[(4, 1, 1, 1, 1)], adjacency=1,
                             entry_point=0)
    assert e.value.status == ann.EINVAL and "even" in str(e.value)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_upload_index(n=10, d=4, degree=2, metric=0, vectors=None, levels=[(8, 1, 1, 1, None)], adjacency=1,
                             entry_point=0)
    assert "norm_term" in str(e.value)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(None, 1, 1, k=1, ef=1, out_ids=1)
    assert e.value.status == ann.EINVAL
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(1, 1, 1, k=10, ef=5, out_ids=1)
    assert "ef" in str(e.value)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(1, 1, 1, k=10, ef=1000, out_ids=1)
    assert e.value.status == ann.ECAPACITY
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(1, 1, 1, k=10, ef=64, out_ids=1, visited_slots=1000)
    assert "power of two" in str(e.value)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(1, 1, 1, k=10, ef=64, out_ids=1, visited_kind=ann.VISITED_TABLE, visited_slots=128)
    assert "minimum" in str(e.value)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(1, 1, 1, k=10, ef=64, out_ids=1, visited_kind=4)
    assert "visited_kind" in str(e.value)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(1, 1, 1, k=10, ef=64, out_ids=1, visited_slots=16384)
    assert e.value.status == ann.ECAPACITY
    with pytest.raises(ann.AnnError) as e:
        ann.ann_search_batch(1, 1, 1, k=10, ef=64, out_ids=1, alpha_s=-1.0)
    assert "alpha_s" in str(e.value)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_bruteforce_topk(1, 100, 8, 1, 1, 300, 0, 1, 1)
    assert e.value.status == ann.ECAPACITY
    with pytest.raises(ann.AnnError) as e:
        ann.ann_sq_encode(1, 10, 5, 4, 1, 1, 1, 1)
    assert e.value.status == ann.EINVAL
    assert ann.ann_version().startswith("ann-gfx950")
