"""The C-ABI library loads, exports every symbol the header declares, and validates arguments
on the host (no kernels run here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "gcada.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(gcada_[a-z_]+)\s*\(", txt)))


def test_exports_match_header():
    from paper_2201_04301_amd import binding as B
    names = _declared()
    assert len(names) >= 11
    for n in names:
        assert hasattr(B.lib, n), n
        assert hasattr(B, n), f"binding lacks {n}"
    assert sorted(B.EXPORTS) == names


def test_create_rejects_bad_arguments_before_touching_a_device():
    from paper_2201_04301_amd import binding as B
    good = dict(G=3, M_G=2, D=10, c=1.0, alpha=1e-2, beta1=0.9, beta2=0.999, eps=1e-8)
    bad_dims = [B.make_dims(7, B.GCADA_F32, [8], 4), B.make_dims(B.GCADA_LOGREG, B.GCADA_BF16, [8], 4),
                B.make_dims(B.GCADA_LOGREG, B.GCADA_F32, [8, 2], 4),
                B.make_dims(B.GCADA_MLP, B.GCADA_F32, [8], 4),
                B.make_dims(B.GCADA_LOGREG, B.GCADA_F32, [0], 4),
                B.make_dims(B.GCADA_LOGREG, B.GCADA_F32, [8], 0),
                B.make_dims(B.GCADA_LOGREG, B.GCADA_F32, [8], 4, l2=-1.0),
                B.make_dims(B.GCADA_MLP, B.GCADA_BF16, [8, 4], 4, l2=1e-3)]
    for d in bad_dims:
        with pytest.raises(B.GcadaError) as e:
            B.gcada_create(d, **good)
        assert e.value.code == B.GCADA_EINVAL
    ok = B.make_dims(B.GCADA_LOGREG, B.GCADA_F32, [8], 4)
    for k, v in [("G", 0), ("M_G", 0), ("D", 0), ("c", -1.0), ("alpha", 0.0), ("beta1", 1.0),
                 ("beta2", -0.1), ("eps", 0.0), ("c", float("nan"))]:
        kw = dict(good)
        kw[k] = v
        with pytest.raises(B.GcadaError) as e:
            B.gcada_create(ok, **kw)
        assert e.value.code == B.GCADA_EINVAL, k
    assert B.lib.gcada_step(None, None, None, None, None) == B.GCADA_EINVAL
    B.gcada_destroy(None)
    assert B.gcada_version().startswith("gcada")
