"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol, and rejects bad
arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2509_09682_amd import binding as B
    from paper_2509_09682_amd import build

    if not os.path.exists(B.LIB_PATH):
        build.build()
    return B


def test_library_exports_every_declared_symbol(binding):
    header = open(os.path.join(ROOT, "include", "cce_neg.h")).read()
    declared = set(re.findall(r"\b(cce_neg_\w+|cce_status_string)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings(binding):
    seen = {binding.status_string(s) for s in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert binding.status_string(99) == "unknown status"


def test_workspace_bytes_rejects_bad_descriptors(binding):
    B = binding
    good = B.make_desc(512, 4096, 64, 128, B.CCE_F32, B.CCE_NEG_SHARED)
    assert B.cce_neg_workspace_bytes(good) >= 256
    for kw in (dict(N=-1), dict(V=0), dict(d=0), dict(d=12), dict(d=520), dict(K=-1), dict(in_dtype=5),
               dict(neg_mode=3), dict(dH_dtype=B.CCE_BF16), dict(algo=9), dict(V=1 << 31)):
        f = dict(N=512, V=4096, d=64, K=128, in_dtype=B.CCE_F32, neg_mode=B.CCE_NEG_SHARED, dH_dtype=B.CCE_F32, algo=0)
        f.update(kw)
        desc = B.make_desc(f["N"], f["V"], f["d"], f["K"], f["in_dtype"], f["neg_mode"], dH_dtype=f["dH_dtype"], algo=f["algo"])
        assert B.cce_neg_workspace_bytes(desc) == 0, kw
    # workspace stays O(N + K d): growing K or N by 10x must not grow it by the product
    a = B.cce_neg_workspace_bytes(B.make_desc(51200, 50000, 64, 1024, B.CCE_BF16, B.CCE_NEG_SHARED))
    b = B.cce_neg_workspace_bytes(B.make_desc(51200, 50000, 64, 10240, B.CCE_BF16, B.CCE_NEG_SHARED))
    c = B.cce_neg_workspace_bytes(B.make_desc(512000, 50000, 64, 10240, B.CCE_BF16, B.CCE_NEG_SHARED))
    assert b <= a + 10240 * 64 * 16 and c <= b + 512000 * 64 * 8
    # per-position mode: the inverted index is built in slices of a fixed pair budget, so ten times the negatives must
    # not cost ten times the workspace, and the index never outgrows 3/8 of the id matrix (4 N K bytes) plus O(N + V)
    def pp(N, V, K, d=128):
        return B.cce_neg_workspace_bytes(B.make_desc(N, V, d, K, B.CCE_BF16, B.CCE_NEG_PER_POSITION))
    c3 = pp(25600, 1_000_000, 256)
    assert c3 <= 12.2 * (1 << 22) + 4 * 1_000_000 + 4 * 25600 + (4 << 20)       # one slice of 2^22 pairs, not 12 N K = 79 MB
    assert pp(25600, 1_000_000, 2560) <= 2.1 * c3
    big = pp(204800, 1_000_000, 2560)                                           # 524 M pairs
    assert big <= 0.375 * 4 * 204800 * 2560 * 1.05 + 4 * 1_000_000 + 4 * 204800 + (34 << 20)
    assert pp(1024, 5_000_000, 16) > 4 * 5_000_000                             # huge catalogue, few pairs: indexed (cursor per item)
    assert pp(204800, 5_000_000, 256) == 256                                    # huge catalogue, many pairs: atomics, header only


def test_forward_backward_reject_null_and_small_workspace_before_launch(binding):
    B = binding
    L = B.lib()
    desc = B.make_desc(16, 100, 64, 8, B.CCE_F32, B.CCE_NEG_SHARED)
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: every call below must fail on the host
    st = L.cce_neg_forward(ctypes.byref(desc), None, fake, fake, fake, None, fake, fake, fake, 4096, None)
    assert st == B.CCE_ERR_NULL
    st = L.cce_neg_forward(ctypes.byref(desc), fake, fake, fake, None, None, fake, fake, fake, 4096, None)
    assert st == B.CCE_ERR_NULL  # K > 0 needs neg
    st = L.cce_neg_forward(ctypes.byref(desc), fake, fake, fake, fake, None, fake, fake, None, 4096, None)
    assert st == B.CCE_ERR_WORKSPACE
    st = L.cce_neg_forward(ctypes.byref(desc), fake, fake, fake, fake, None, fake, fake, fake, 8, None)
    assert st == B.CCE_ERR_WORKSPACE
    st = L.cce_neg_forward(ctypes.byref(desc), fake, fake, fake, fake, None, fake, fake, ctypes.c_void_p(0x1004), 4096, None)
    assert st == B.CCE_ERR_WORKSPACE  # misaligned
    st = L.cce_neg_forward(ctypes.byref(desc), fake, fake, fake, fake, None, None, fake, fake, 4096, None)
    assert st == B.CCE_ERR_NULL
    st = L.cce_neg_backward(ctypes.byref(desc), fake, fake, fake, fake, None, None, None, fake, fake, fake, 4096, None)
    assert st == B.CCE_ERR_NULL  # lse missing
    st = L.cce_neg_backward(ctypes.byref(desc), fake, fake, fake, fake, None, fake, None, fake, None, fake, 4096, None)
    assert st == B.CCE_ERR_NULL  # dE missing
    bad = B.make_desc(16, 100, 60, 8, B.CCE_F32, B.CCE_NEG_SHARED)
    st = L.cce_neg_forward(ctypes.byref(bad), fake, fake, fake, fake, None, fake, fake, fake, 4096, None)
    assert st == B.CCE_ERR_SHAPE
    bad = B.make_desc(16, 100, 64, 8, B.CCE_F32, B.CCE_NEG_SHARED, dH_dtype=B.CCE_BF16)
    st = L.cce_neg_backward(ctypes.byref(bad), fake, fake, fake, fake, None, fake, None, fake, fake, fake, 4096, None)
    assert st == B.CCE_ERR_DTYPE
    assert L.cce_neg_workspace_init(None, 4096, None) == B.CCE_ERR_NULL
    assert L.cce_neg_index_status(None, 4096, None) == B.CCE_ERR_NULL


def test_gradient_filtering_is_accepted_only_where_it_is_defined(binding):
    B = binding
    ok = B.make_desc(256, 1000, 64, 0, B.CCE_BF16, B.CCE_NEG_FULL, filter_eps=1e-4)
    assert B.cce_neg_workspace_bytes(ok) > 0
    for kw in (dict(neg_mode=B.CCE_NEG_SHARED, K=64, in_dtype=B.CCE_BF16, d=64),   # sampled modes do not filter (Sec. 3.3)
               dict(neg_mode=B.CCE_NEG_FULL, K=0, in_dtype=B.CCE_F32, d=64),       # fp32 runs on the row-gather path
               dict(neg_mode=B.CCE_NEG_FULL, K=0, in_dtype=B.CCE_BF16, d=96)):     # no matrix-core kernel for this d
        desc = B.make_desc(256, 1000, kw["d"], kw["K"], kw["in_dtype"], kw["neg_mode"], filter_eps=1e-4)
        assert B.cce_neg_workspace_bytes(desc) == 0
    for bad in (-1.0, float("nan")):
        assert B.cce_neg_workspace_bytes(B.make_desc(256, 1000, 64, 0, B.CCE_BF16, B.CCE_NEG_FULL, filter_eps=bad)) == 0


def test_sampled_calls_reject_bad_samplers_before_launch(binding):
    B = binding
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)  # never dereferenced
    desc = B.make_desc(16, 100, 64, 8, B.CCE_F32, B.CCE_NEG_PER_POSITION)
    ok = B.make_sampler(B.CCE_SAMPLER_UNIFORM, 1, 0)
    assert L.cce_neg_sample(ctypes.byref(desc), None, fake, None) == B.CCE_ERR_NULL
    assert L.cce_neg_sample(ctypes.byref(desc), ctypes.byref(ok), None, None) == B.CCE_ERR_NULL
    assert L.cce_neg_sample(ctypes.byref(desc), ctypes.byref(B.make_sampler(7, 1, 0)), fake, None) == B.CCE_ERR_SHAPE
    alias_without_table = B.make_sampler(B.CCE_SAMPLER_ALIAS, 1, 0)
    assert L.cce_neg_sample(ctypes.byref(desc), ctypes.byref(alias_without_table), fake, None) == B.CCE_ERR_NULL
    full = B.make_desc(16, 100, 64, 0, B.CCE_F32, B.CCE_NEG_FULL)
    assert L.cce_neg_sample(ctypes.byref(full), ctypes.byref(ok), fake, None) == B.CCE_ERR_UNSUPPORTED
    big = 1 << 30
    st = L.cce_neg_forward_sampled(ctypes.byref(full), ctypes.byref(ok), fake, fake, fake, None, fake, fake, fake, big, None)
    assert st == B.CCE_ERR_UNSUPPORTED
    st = L.cce_neg_forward_sampled(ctypes.byref(desc), ctypes.byref(ok), fake, fake, None, None, fake, fake, fake, big, None)
    assert st == B.CCE_ERR_NULL   # tgt missing
    st = L.cce_neg_forward_sampled(ctypes.byref(desc), ctypes.byref(ok), fake, fake, fake, None, fake, fake, fake, 8, None)
    assert st == B.CCE_ERR_WORKSPACE
    st = L.cce_neg_backward_sampled(ctypes.byref(desc), ctypes.byref(ok), fake, fake, fake, None, None, None, fake, fake,
                                    fake, big, None)
    assert st == B.CCE_ERR_NULL   # lse missing
    st = L.cce_neg_backward_sampled(ctypes.byref(desc), ctypes.byref(alias_without_table), fake, fake, fake, None, fake,
                                    None, fake, fake, fake, big, None)
    assert st == B.CCE_ERR_NULL
    # the shared list the sampled calls draw has its corner of the workspace
    a = B.cce_neg_workspace_bytes(B.make_desc(512, 4096, 64, 128, B.CCE_F32, B.CCE_NEG_SHARED))
    b = B.cce_neg_workspace_bytes(B.make_desc(512, 4096, 64, 1024, B.CCE_F32, B.CCE_NEG_SHARED))
    assert b - a >= (1024 - 128) * 4


def test_binding_refuses_wrong_dtypes_and_shapes_before_any_launch(binding):
    """The C ABI reads raw bytes: a torch.long index tensor, a short mask or a mis-shaped per-position `neg` must be
    refused by the binding (and so by cce_neg_loss) before a pointer is formed.  CPU tensors suffice: a call that got
    past the checks would stop at the CUDA-tensor requirement, with another message."""
    import torch

    B = binding
    N, V, d, K = 6, 50, 16, 4
    desc = B.make_desc(N, V, d, K, B.CCE_F32, B.CCE_NEG_PER_POSITION)
    H, E = torch.zeros(N, d), torch.zeros(V, d)
    tgt = torch.zeros(N, dtype=torch.int32)
    neg = torch.zeros(N, K, dtype=torch.int32)
    mask = torch.ones(N, dtype=torch.uint8)
    loss, lse = torch.zeros(N), torch.zeros(N)
    ws = torch.zeros(1 << 16, dtype=torch.uint8)

    def fwd(**kw):
        a = dict(H=H, E=E, tgt=tgt, neg=neg, mask=mask, loss=loss, lse=lse)
        a.update(kw)
        return B.cce_neg_forward(desc, a["H"], a["E"], a["tgt"], a["neg"], a["mask"], a["loss"], a["lse"], ws)

    with pytest.raises(TypeError, match="tgt"):
        fwd(tgt=tgt.long())
    with pytest.raises(TypeError, match="neg"):
        fwd(neg=neg.long())
    with pytest.raises(TypeError, match="mask"):
        fwd(mask=mask.float())
    with pytest.raises(TypeError, match="H"):
        fwd(H=H.double())
    with pytest.raises(ValueError, match="tgt"):
        fwd(tgt=tgt[:-1])
    with pytest.raises(ValueError, match="mask"):
        fwd(mask=mask[:-1])
    with pytest.raises(ValueError, match="neg"):
        fwd(neg=neg[:, :-1])
    with pytest.raises(ValueError, match="neg"):
        fwd(neg=neg.t().contiguous())          # [K, N]: right size, wrong shape
    with pytest.raises(ValueError, match="neg"):
        fwd(neg=None)
    with pytest.raises(ValueError, match="E"):
        fwd(E=E[:-1])
    with pytest.raises(ValueError, match="CUDA"):   # well-formed arguments get as far as the device-pointer requirement
        fwd()
    g, dH, dE = torch.zeros(N), torch.zeros(N, d), torch.zeros(V, d)
    with pytest.raises(TypeError, match="dE"):
        B.cce_neg_backward(desc, H, E, tgt, neg, mask, lse, g, dH, dE.double(), ws)
    with pytest.raises(TypeError, match="dH"):
        B.cce_neg_backward(desc, H, E, tgt, neg, mask, lse, g, dH.bfloat16(), dE, ws)
    with pytest.raises(ValueError, match="grad_loss"):
        B.cce_neg_backward(desc, H, E, tgt, neg, mask, lse, g[:-1], dH, dE, ws)
    bad_mode = B.make_desc(N, V, d, K, B.CCE_F32, 7)
    with pytest.raises(ValueError, match="neg_mode"):
        B.cce_neg_forward(bad_mode, H, E, tgt, neg, mask, loss, lse, ws)
    # the autograd front end goes through the same checks
    from paper_2509_09682_amd import cce_neg_loss

    with pytest.raises(TypeError, match="tgt"):
        cce_neg_loss(H, E, tgt.long(), neg, mask, neg_mode=B.CCE_NEG_PER_POSITION)
