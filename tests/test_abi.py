"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(rabitq_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_named_calls():
    d = _declared()
    assert "rabitq_index_upload" in d and "rabitq_search" in d and len(d) >= 12


def test_library_exports_every_declared_symbol():
    from paper_2602_23999_amd import rabitq
    if not os.path.exists(rabitq.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    lib = ctypes.CDLL(rabitq.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(rabitq.EXPORTS) == _declared()


def test_binding_fails_loudly_without_a_device():
    import torch
    from paper_2602_23999_amd import rabitq
    if torch.cuda.is_available():
        pytest.skip("a device is present")
    import numpy as np
    with pytest.raises(rabitq.RabitqError):
        rabitq.Index(dim=32, nlist=1, n=0, total_bits=1, metric="l2", rotation=np.eye(32), centroids=np.zeros((1, 32)),
                     offsets=np.zeros(2), short_codes=np.zeros(0), short_factors=np.zeros(0), ids=np.zeros(0))


def test_host_side_argument_errors_need_no_device():
    from paper_2602_23999_amd import rabitq
    lib = rabitq.load_library()
    assert lib.rabitq_index_upload(None, None, None) == -1
    assert b"null" in lib.rabitq_last_error()
    assert lib.rabitq_search(None, None, 1, 1, 1, None, None, None) == -1
    assert lib.rabitq_probe_list_scratch_words(1024, 10000) == 2 * 1024 * 313 + 1024
    assert lib.rabitq_index_free(None) == 0
    # a dimension without scan kernels is rejected before anything touches the device
    desc = rabitq._Desc(160, 4, 0, 1, 0, None, None, None, None, None, None, None, None, None)
    h = ctypes.c_void_p()
    assert lib.rabitq_index_upload(ctypes.byref(desc), ctypes.byref(h), None) == -1
    assert b"dim must be one of" in lib.rabitq_last_error()
    prm = rabitq._BuildParams(1536, 4, 0, 1, 0, 1, 0, 1.9, None, 0)
    assert lib.rabitq_index_build(ctypes.byref(prm), None, ctypes.byref(h), None) == -1
    assert b"dim must be one of" in lib.rabitq_last_error()


def _header_structs():
    """name -> member names, for every `typedef struct { ... } name;` of the headers."""
    out = {}
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            for body, name in re.findall(r"typedef\s+struct\s*\{(.*?)\}\s*(\w+)\s*;", text, flags=re.S):
                members = []
                for decl in body.split(";"):
                    decl = decl.strip()
                    if decl:  # "type a, b" declares two members
                        members += [re.findall(r"(\w+)\s*$", part.strip())[0] for part in decl.split(",")]
                out[name] = members
    return out


def test_binding_structures_match_the_header_member_for_member():
    # a binding structure shorter than the header's makes the library read past its end
    from paper_2602_23999_amd import rabitq
    structs = _header_structs()
    for cname, ctype in (("rabitq_query_repr", rabitq._QueryRepr), ("rabitq_index_desc", rabitq._Desc),
                         ("rabitq_build_params", rabitq._BuildParams)):
        assert [f[0] for f in ctype._fields_] == structs[cname], cname
    assert ctypes.sizeof(rabitq._QueryRepr) == 8 * len(structs["rabitq_query_repr"])


def test_stream_probe_driver_is_built_and_links_against_the_library():
    """The stand-alone driver of the streaming-regime scan (csrc/stream_probe.hip) is built beside the library and
    finds it through its run path; with arguments out of range it prints its usage before any GPU call."""
    import subprocess
    from paper_2602_23999_amd import rabitq
    exe = os.path.join(os.path.dirname(rabitq.LIB_PATH), "stream_probe")
    assert os.path.exists(exe), "run __graft_entry__.build()"
    r = subprocess.run([exe, "1"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=60)
    assert r.returncode == 1 and "usage: stream_probe" in r.stdout
