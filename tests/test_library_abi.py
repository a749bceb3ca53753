"""The C-ABI library loads and exports every symbol the public header declares; host-side argument
checks answer with error codes before anything touches a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "dsbd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dsbd_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    import paper_2409_16560_amd as dsbd
    lib = dsbd.load_library()
    names = header_functions()
    assert {"dsbd_forest_attention", "dsbd_verify_forest", "dsbd_select_beams", "dsbd_commit_kv", "dsbd_draft_layer",
            "dsbd_build_forest"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in dsbd.dsbd_version()


def test_binding_structs_match_header_field_order():
    import paper_2409_16560_amd.binding as b
    src = open(os.path.join(ROOT, "include", "dsbd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    for cname, cls in (("dsbd_forest", b._Forest), ("dsbd_kv", b._KV), ("dsbd_params", b._Params),
                       ("dsbd_verify_in", b._VerifyIn), ("dsbd_verify_out", b._VerifyOut),
                       ("dsbd_next_beams", b._NextBeams), ("dsbd_kv_dst", b._KVDst), ("dsbd_draft_in", b._DraftIn),
                       ("dsbd_draft_out", b._DraftOut), ("dsbd_forest_out", b._ForestOut)):
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (cname, cname), src, flags=re.S).group(1)
        fields = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            names = decl.split(",")
            first = re.findall(r"([A-Za-z_][A-Za-z_0-9]*)\s*$", names[0].strip())[0]
            fields.append(first)
            for extra in names[1:]:
                fields.append(re.findall(r"([A-Za-z_][A-Za-z_0-9]*)\s*$", extra.strip())[0])
        assert fields == [n for n, _ in cls._fields_], cname


def test_host_side_argument_checks_need_no_gpu():
    import paper_2409_16560_amd.binding as b
    lib = b.load_library()
    f = b._Forest(1, 1, 3, None, None, None, None, None, 3, 2, 1)
    kv = b._KV(None, None, None, None, None, None, 128, 64, 16)
    # Hq not a multiple of Hkv -> invalid; D = 96 -> unsupported; 65-node trees -> unsupported
    assert lib.dsbd_forest_attention(C.byref(f), C.byref(kv), None, None, None, 6, 4, 128, 0.0, None, None, None, None, 0, None, None) == -1
    assert lib.dsbd_forest_attention(C.byref(f), C.byref(kv), None, None, None, 8, 4, 96, 0.0, None, None, None, None, 0, None, None) == -2
    f65 = b._Forest(1, 1, 65, None, None, None, None, None, 65, 2, 1)
    assert lib.dsbd_forest_attention(C.byref(f65), C.byref(kv), None, None, None, 8, 4, 128, 0.0, None, None, None, None, 0, None, None) == -2
    assert lib.dsbd_forest_attention_workspace_bytes(C.byref(f65), C.byref(kv), 8, 4, 128) == 0
    # null array pointers with a non-empty forest -> invalid
    assert lib.dsbd_forest_attention(C.byref(f), C.byref(kv), None, None, None, 8, 4, 128, 0.0, None, None, None, None, 0, None, None) == -1
    p = b._Params(4, 1, 2, -1.0)      # W_L above W_cap
    assert lib.dsbd_verify_forest_workspace_bytes(C.byref(f), 100, C.byref(p)) == 0
    p = b._Params(2, 1, 4, -1.0)
    assert lib.dsbd_verify_forest_workspace_bytes(C.byref(f), 0, C.byref(p)) == 0     # V < 1
    assert lib.dsbd_verify_forest_workspace_bytes(C.byref(f), 100, C.byref(p)) > 0
    for top_k, top_p in ((33, 1.0), (0, 0.5), (-1, 1.0), (4, -0.5)):      # warping outside what is supported
        pw = b._Params(2, 1, 4, -1.0, top_k, top_p)
        assert lib.dsbd_verify_forest_workspace_bytes(C.byref(f), 100, C.byref(pw)) == 0
    pw = b._Params(2, 1, 4, -1.0, 32, 0.9)
    assert lib.dsbd_verify_forest_workspace_bytes(C.byref(f), 100, C.byref(pw)) > 0
    # a threshold that is not a number must not slip through as "dynamic width" (NaN compares false with everything)
    pn = b._Params(2, 1, 4, float("nan"))
    assert lib.dsbd_verify_forest_workspace_bytes(C.byref(f), 100, C.byref(pn)) == 0
    assert lib.dsbd_verify_forest_workspace_bytes(C.byref(f), 100, C.byref(b._Params(2, 1, 4, 1.5))) == 0
    vin = b._VerifyIn(100, None, None, None, None, None, None, None)
    vout = b._VerifyOut(*([None] * 14))
    assert lib.dsbd_verify_forest(C.byref(f), C.byref(vin), C.byref(p), C.byref(vout), None, 0, None, None) == -1
    nb = b._NextBeams(*([None] * 8))
    assert lib.dsbd_select_beams(C.byref(f), C.byref(vout), 4, 0, C.byref(nb), None, None) == -1
    assert lib.dsbd_select_beams(C.byref(f), C.byref(vout), 65, 0, C.byref(nb), C.c_void_p(8), None) == -2
    kd = b._KVDst(None, None, None, 16)
    assert lib.dsbd_commit_kv(C.byref(f), C.byref(kv), None, None, 8, 128, C.byref(nb), 4, C.byref(kd), None, None) == -1
    assert lib.dsbd_commit_kv(C.byref(f), C.byref(kv), None, None, 8, 100, C.byref(nb), 4, C.byref(kd), C.c_void_p(8), None) == -2
    assert lib.dsbd_commit_kv(C.byref(f), C.byref(kv), None, None, 8, 128, C.byref(nb), 4, C.byref(kd), C.c_void_p(8), None) == -1
    di = b._DraftIn(1, 2, 2, 100, None, None, None, None)
    do = b._DraftOut(None, None, None)
    assert lib.dsbd_draft_layer_workspace_bytes(C.byref(di), 4, 0, 1.0) > 0
    assert lib.dsbd_draft_layer_workspace_bytes(C.byref(di), 65, 0, 1.0) == 0          # W_S above 64
    assert lib.dsbd_draft_layer_workspace_bytes(C.byref(di), 4, 33, 1.0) == 0          # top_k above 32
    assert lib.dsbd_draft_layer(C.byref(di), 4, 0, 1.0, C.byref(do), None, 0, C.c_void_p(8), None) == -1   # null arrays
    assert lib.dsbd_draft_layer(C.byref(di), 0, 0, 1.0, C.byref(do), None, 0, C.c_void_p(8), None) == -2
    fo = b._ForestOut(*([None] * 8))
    assert lib.dsbd_build_forest(1, 2, 3, 4, None, None, None, None, C.byref(fo), C.c_void_p(8), None) == -1
    assert lib.dsbd_build_forest(1, 2, 3, 65, None, None, None, None, C.byref(fo), C.c_void_p(8), None) == -2
    assert lib.dsbd_build_forest(0, 0, 0, 0, None, None, None, None, C.byref(fo), C.c_void_p(8), None) == 0


def test_workspace_sizes_scale_with_the_problem():
    import paper_2409_16560_amd.binding as b
    lib = b.load_library()
    kv = b._KV(None, None, None, None, None, None, 1024, 128, 8192)
    small = b._Forest(1, 2, 6, None, None, None, None, None, 3, 2, 2)
    big = b._Forest(1, 8, 248, None, None, None, None, None, 31, 4, 8)
    a = lib.dsbd_forest_attention_workspace_bytes(C.byref(small), C.byref(kv), 32, 8, 128)
    c = lib.dsbd_forest_attention_workspace_bytes(C.byref(big), C.byref(kv), 32, 8, 128)
    assert 0 < a < c
    p = b._Params(0, 1, 16, 0.9)
    assert 0 < lib.dsbd_verify_forest_workspace_bytes(C.byref(small), 256, C.byref(p)) < \
        lib.dsbd_verify_forest_workspace_bytes(C.byref(big), 128256, C.byref(p))


def test_prefix_kv_refuses_caches_of_different_strides():
    """One token stride and one head stride serve all caches (include/dsbd.h, dsbd_kv): head-major tensors of
    different lengths would be read out of bounds, so the binding refuses them; views of equally sized buffers pass."""
    import torch
    import paper_2409_16560_amd as dsbd
    k = [torch.zeros(4, 10, 64, dtype=torch.bfloat16), torch.zeros(4, 20, 64, dtype=torch.bfloat16)]
    with pytest.raises(ValueError):
        dsbd.PrefixKV(k, k, head_major=True)
    buf = [torch.zeros(4, 32, 64, dtype=torch.bfloat16) for _ in range(2)]
    views = [buf[0][:, :10], buf[1][:, :20]]
    kv = dsbd.PrefixKV(views, views, head_major=True)
    assert (kv.token_stride, kv.head_stride, kv.max_len) == (64, 32 * 64, 20)
    k = [torch.zeros(10, 4, 64, dtype=torch.bfloat16), torch.zeros(20, 4, 64, dtype=torch.bfloat16)]
    kv = dsbd.PrefixKV(k, k)
    assert (kv.token_stride, kv.head_stride) == (256, 64)
    with pytest.raises(ValueError):
        dsbd.PrefixKV(k, [k[0], torch.zeros(20, 8, 64, dtype=torch.bfloat16)])
