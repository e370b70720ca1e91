"""The C-ABI library: it loads without a GPU, exports every symbol the header declares,
and its host-side logic (sizes, rounding, validation) behaves as documented. No kernel runs here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    if not os.path.exists(os.path.join(ROOT, "paper_2604_06694_amd", "libaudiokv.so")):
        from paper_2604_06694_amd import build
        build.build()
    return A


def declared_functions():
    text = open(os.path.join(ROOT, "include", "audiokv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(audiokv_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(A):
    names = declared_functions()
    assert {"audiokv_score", "audiokv_allocate", "audiokv_smooth", "audiokv_select", "audiokv_compact",
            "audiokv_evict"} <= set(names)
    lib = C.CDLL(A.lib_path())
    for n in names:
        assert hasattr(lib, n), n


def test_n_keep_matches_oracle_rounding(A):
    from oracle import audiokv_oracle as O
    rng = np.random.default_rng(0)
    for _ in range(2000):
        L = int(rng.integers(1, 70000))
        r = float(rng.uniform(0.01, 1.0))
        assert A.n_keep(r, L) == O.n_keep_of(r, L)
    for r, L in [(0.4, 2048), (0.2, 32768), (0.4, 32768), (0.3, 5003), (0.5, 5), (0.25, 10)]:
        assert A.n_keep(r, L) == O.n_keep_of(r, L)
    assert A.n_keep(0.4, 2048) == 819 and A.n_keep(0.4, 32768) == 13107 and A.n_keep(0.2, 32768) == 6554


def test_total_kept_and_workspace(A):
    p = A.Params(28, 4, 128, 64)
    assert A.total_kept(p, [32768] * 28, 0.4) == 13107 * 4 * 28
    assert A.total_kept(A.Params(8, 2, 256, 32), [2048, 5000], 0.3) == (614 + 1500) * 2
    small = A.workspace_bytes(p, [4096])
    big = A.workspace_bytes(p, [32768] * 28)
    assert 0 < small < big
    assert big >= 2 * 28 * 4 * 32768 * 4          # raw + smoothed scores


def test_validation_errors_are_codes_not_crashes(A):
    good = A.Params(28, 4, 128, 32)
    cases = [
        (A.Params(28, 5, 128, 32), -1),           # H_q not a multiple of H_kv
        (A.Params(28, 4, 96, 32), -2),            # head_dim not built
        (A.Params(28, 4, 128, 32, pool_kernel=4), -1),
        (A.Params(28, 4, 128, 32, floor_frac=1.5), -1),
        (A.Params(28, 4, 128, 32, kv_layout=7), -1),
        # explicit K/V strides: rows are moved as 16-byte vectors and may not overlap within a head
        (A.Params(28, 4, 128, 32, kv_stride_head=4096 * 128, kv_stride_tok=132), -1),     # token stride not a multiple of 8
        (A.Params(28, 4, 128, 32, kv_stride_head=4096 * 128 + 4, kv_stride_tok=128), -1), # head stride not a multiple of 8
        (A.Params(28, 4, 128, 32, kv_stride_head=4096 * 128, kv_stride_tok=64), -1),      # token stride below head_dim
        (A.Params(28, 4, 128, 32, kv_stride_tok=128), -1),                                # head stride missing
        (A.Params(28, 4, 128, 32, kv_stride_item=-8, kv_stride_head=4096 * 128, kv_stride_tok=128), -1),
    ]
    for p, code in cases:
        with pytest.raises(A.AudioKVError) as e:
            A.workspace_bytes(p, [2048])
        assert e.value.code == code
    strided = A.Params(28, 4, 128, 32, kv_stride_head=4096 * 128, kv_stride_tok=128)
    assert A.workspace_bytes(strided, [2048]) == A.workspace_bytes(good, [2048])      # one item: no item stride needed
    with pytest.raises(A.AudioKVError) as e:
        A.workspace_bytes(strided, [2048, 1000])  # several items need kv_stride_item
    assert e.value.code == -1
    with pytest.raises(A.AudioKVError) as e:
        A.total_kept(good, [2048], 0.001)         # n_keep below the window
    assert e.value.code == -1
    with pytest.raises(A.AudioKVError) as e:
        A.total_kept(good, [16], 0.5)             # L below the window
    assert e.value.code == -1
    # a GPU entry point given NULL pointers returns before touching the device
    lib = A.binding._lib
    cp = good.c()
    lens = (C.c_int32 * 1)(2048)
    rc = lib.audiokv_score(C.byref(cp), None, None, None, lens, 1, None, None, 0, None)
    assert rc == -1 and b"NULL" in lib.audiokv_last_error()
    rc = lib.audiokv_evict(C.byref(cp), None, None, None, None, 1, None, lens, 1, 0.4, 0.125, 1.0,
                           None, None, None, None, None, None, 0, None)
    assert rc == -1
    bad = A.Params(28, 4, 128, 32).c()
    bad.size = 12
    rc = lib.audiokv_score(C.byref(bad), None, None, None, lens, 1, None, None, 0, None)
    assert rc == -1 and b"size" in lib.audiokv_last_error()


def test_empty_batch_is_accepted_everywhere_and_enqueues_nothing(A):
    """n_items = 0: every entry point returns AUDIOKV_OK before looking at any pointer (so this runs without a GPU);
    sizes come back as 0. Invalid params are still refused."""
    p = A.Params(28, 4, 128, 32)
    assert A.total_kept(p, [], 0.4) == 0
    assert A.workspace_bytes(p, []) == 0
    lib = A.binding._lib
    cp = p.c()
    assert lib.audiokv_score(C.byref(cp), None, None, None, None, 0, None, None, 0, None) == 0
    assert lib.audiokv_score_lse(C.byref(cp), None, None, None, None, None, 0, None, None, 0, None) == 0
    assert lib.audiokv_allocate(C.byref(cp), None, 0, 4, 1, None, None, C.c_double(0.4), None, None, None) == 0
    assert lib.audiokv_smooth(C.byref(cp), None, None, None, 0, C.c_double(0.125), C.c_double(1.0), None, None, 0, None) == 0
    assert lib.audiokv_smooth_cutoffs(C.byref(cp), None, None, None, 0, C.c_double(0.9), None, None, 0, None) == 0
    assert lib.audiokv_select(C.byref(cp), None, None, None, None, None, 0, None, None, 0, None) == 0
    assert lib.audiokv_compact(C.byref(cp), None, None, None, None, None, None, 0, C.c_int64(0), None, None, None) == 0
    assert lib.audiokv_evict(C.byref(cp), None, None, None, None, 1, None, None, 0, C.c_double(0.4), C.c_double(0.125),
                             C.c_double(1.0), None, None, None, None, None, None, 0, None) == 0
    out = C.c_size_t(7)
    assert lib.audiokv_decode_workspace_bytes(C.byref(cp), 0, C.c_int64(0), C.byref(out)) == 0 and out.value == 0
    assert lib.audiokv_decode_attend(C.byref(cp), None, None, None, None, 0, C.c_int64(0), None, None, 0, None) == 0
    bad = A.Params(28, 5, 128, 32).c()
    assert lib.audiokv_evict(C.byref(bad), None, None, None, None, 1, None, None, 0, C.c_double(0.4), C.c_double(0.125),
                             C.c_double(1.0), None, None, None, None, None, None, 0, None) == -1
