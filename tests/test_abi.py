"""The C-ABI library loads, exports what include/dynadiag.h declares, and rejects bad arguments
on the host before anything touches a GPU (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2506_11449_amd as dd
from paper_2506_11449_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dynadiag.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_11449_amd.build import build_library
        build_library()
    return dd.load_library()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    assert lib.dd_status_string(0) == b"ok"
    assert {lib.dd_status_string(i) for i in range(5)}.__len__() == 5


def _layer(T=4, M=8, N=8, K=2, dtype=0, algo=0):
    return binding.dd_layer(T, M, N, K, dtype, algo)


def test_invalid_arguments_are_rejected_on_the_host(lib):
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)  # never dereferenced: every call below fails its host-side checks first
    bad_layers = [_layer(T=-1), _layer(M=0), _layer(N=0), _layer(K=0), _layer(K=9), _layer(dtype=7), _layer(algo=9)]
    for l in bad_layers:
        assert lib.dd_fwd(ctypes.byref(l), one, one, one, one, null, 0, null) == 1
        assert lib.dd_bwd_input(ctypes.byref(l), one, one, one, one, null, 0, null) == 1
        assert lib.dd_bwd_weight(ctypes.byref(l), one, one, one, one, null, 0, null) == 1
        assert lib.dd_workspace_bytes(0, ctypes.byref(l), 0) == 0
    ok = _layer()
    assert lib.dd_fwd(None, one, one, one, one, null, 0, null) == 1
    assert lib.dd_fwd(ctypes.byref(ok), null, one, one, one, null, 0, null) == 1
    assert lib.dd_fwd(ctypes.byref(ok), one, null, one, one, null, 0, null) == 1
    assert lib.dd_fwd(ctypes.byref(ok), one, one, null, one, null, 0, null) == 1
    assert lib.dd_fwd(ctypes.byref(ok), one, one, one, null, null, 0, null) == 1
    assert lib.dd_bwd_weight(ctypes.byref(ok), one, one, one, null, null, 0, null) == 1
    # too wide for the kernels' index types
    assert lib.dd_fwd(ctypes.byref(_layer(M=70000, N=8)), one, one, one, one, null, 0, null) == 2
    # selection
    assert lib.dd_select_diagonals(1, 8, 0, one, one, null, 0, null) == 1
    assert lib.dd_select_diagonals(1, 8, 9, one, one, null, 0, null) == 1
    assert lib.dd_select_diagonals(-1, 8, 2, one, one, null, 0, null) == 1
    assert lib.dd_select_diagonals(1, 8, 2, null, one, null, 0, null) == 1
    assert lib.dd_select_diagonals(1, 1 << 20, 2, one, one, null, 0, null) == 2
    assert lib.dd_select_diagonals(0, 8, 2, null, null, null, 0, null) == 0


def test_workspace_rules(lib):
    l = _layer(T=5000, M=64, N=64, K=8, dtype=1)
    need = lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT, ctypes.byref(l), 0)
    assert need > 0
    one = ctypes.c_void_p(256)
    # missing, short and misaligned workspaces are refused before any launch
    assert lib.dd_bwd_weight(ctypes.byref(l), one, one, one, one, None, 0, None) == 3
    assert lib.dd_bwd_weight(ctypes.byref(l), one, one, one, one, ctypes.c_void_p(512), need - 1, None) == 3
    assert lib.dd_bwd_weight(ctypes.byref(l), one, one, one, one, ctypes.c_void_p(513), need, None) == 3
    # zero tokens need no launch and no buffers for the products
    z = _layer(T=0)
    assert lib.dd_fwd(ctypes.byref(z), None, one, one, None, None, 0, None) == 0
    assert lib.dd_bwd_input(ctypes.byref(z), None, one, one, None, None, 0, None) == 0


def test_prepare_rules(lib):
    one = ctypes.c_void_p(256)
    ok = _layer(T=100, M=768, N=3072, K=30, dtype=1, algo=binding.DD_ALGO_PREPARED)
    need = lib.dd_workspace_bytes(binding.DD_OP_PREPARE, ctypes.byref(ok), 0)
    assert need == 2 * 768 * 3072 * 2  # both dense operands, bf16
    # the prepared calls want the whole block, whatever the density
    assert lib.dd_workspace_bytes(binding.DD_OP_FWD, ctypes.byref(ok), 0) == need
    assert lib.dd_workspace_bytes(binding.DD_OP_BWD_INPUT, ctypes.byref(ok), 0) == need
    assert lib.dd_prepare(ctypes.byref(ok), None, one, one, need, None) == 1
    assert lib.dd_prepare(ctypes.byref(ok), one, None, one, need, None) == 1
    assert lib.dd_prepare(ctypes.byref(ok), one, one, None, need, None) == 3
    assert lib.dd_prepare(ctypes.byref(ok), one, one, ctypes.c_void_p(512), need - 1, None) == 3
    assert lib.dd_prepare(ctypes.byref(ok), one, one, ctypes.c_void_p(520), need, None) == 3
    # shapes and types the matrix-core kernels do not cover
    for bad in (_layer(M=768, N=768, K=8, dtype=0, algo=binding.DD_ALGO_PREPARED),
                _layer(M=100, N=768, K=8, dtype=1, algo=binding.DD_ALGO_PREPARED),
                _layer(M=768, N=768, K=8, dtype=1, algo=binding.DD_ALGO_VECTOR)):
        assert lib.dd_workspace_bytes(binding.DD_OP_PREPARE, ctypes.byref(bad), 0) in (0, 2 * 768 * 768 * 2)
        assert lib.dd_prepare(ctypes.byref(bad), one, one, ctypes.c_void_p(512), 1 << 30, None) == 2
    unsupported = _layer(T=8, M=100, N=768, K=8, dtype=1, algo=binding.DD_ALGO_PREPARED)
    assert lib.dd_fwd(ctypes.byref(unsupported), one, None, None, one, ctypes.c_void_p(512), 1 << 30, None) == 2
    # a prepared product does not read offsets / values, but still needs its block
    assert lib.dd_fwd(ctypes.byref(ok), one, None, None, one, None, 0, None) == 3
    assert lib.dd_bwd_input(ctypes.byref(ok), one, None, None, one, ctypes.c_void_p(512), need - 1, None) == 3


def test_feature_count_limit(lib):
    one = ctypes.c_void_p(256)
    widest = _layer(T=2, M=65535, N=8, K=3)
    too_wide = _layer(T=2, M=65536, N=8, K=3)
    assert lib.dd_workspace_bytes(binding.DD_OP_FWD, ctypes.byref(too_wide), 0) == 0
    for fn in (lib.dd_fwd, lib.dd_bwd_input):
        assert fn(ctypes.byref(too_wide), one, one, one, one, None, 0, None) == 2
        assert fn(ctypes.byref(widest), None, one, one, one, None, 0, None) == 1   # accepted up to the null pointer
    assert lib.dd_bwd_weight(ctypes.byref(too_wide), one, one, one, one, None, 0, None) == 2


def test_select_prepare_rules(lib):
    one = ctypes.c_void_p(256)
    blk = ctypes.c_void_p(512)
    ok = _layer(T=0, M=768, N=768, K=30, dtype=1)
    need = lib.dd_workspace_bytes(binding.DD_OP_PREPARE, ctypes.byref(ok), 0)
    assert lib.dd_select_prepare(ctypes.byref(ok), None, one, one, blk, need, None) == 1
    assert lib.dd_select_prepare(ctypes.byref(ok), one, None, one, blk, need, None) == 1
    assert lib.dd_select_prepare(ctypes.byref(ok), one, one, None, blk, need, None) == 1
    assert lib.dd_select_prepare(ctypes.byref(ok), one, one, one, None, need, None) == 3
    assert lib.dd_select_prepare(ctypes.byref(ok), one, one, one, blk, need - 1, None) == 3
    for bad in (_layer(M=768, N=768, K=8, dtype=0), _layer(M=100, N=768, K=8, dtype=1),
                _layer(M=768, N=768, K=8, dtype=1, algo=binding.DD_ALGO_VECTOR)):
        assert lib.dd_select_prepare(ctypes.byref(bad), one, one, one, blk, 1 << 30, None) == 2
    assert lib.dd_select_prepare(ctypes.byref(_layer(M=768, N=768, K=800, dtype=1)), one, one, one, blk, need, None) == 1


def test_shared_input_rules(lib):
    one = ctypes.c_void_p(256)
    blk = ctypes.c_void_p(512)
    ok = _layer(T=100, M=768, N=768, K=30, dtype=1)
    per_set = lib.dd_workspace_bytes(binding.DD_OP_PREPARE, ctypes.byref(ok), 0)
    assert per_set == 2 * 768 * 768 * 2
    assert lib.dd_prepare_shared(ctypes.byref(ok), 0, one, one, blk, 8 * per_set, None) == 1
    assert lib.dd_prepare_shared(ctypes.byref(ok), 9, one, one, blk, 9 * per_set, None) == 2
    assert lib.dd_prepare_shared(ctypes.byref(ok), 3, None, one, blk, 3 * per_set, None) == 1
    assert lib.dd_prepare_shared(ctypes.byref(ok), 3, one, None, blk, 3 * per_set, None) == 1
    assert lib.dd_prepare_shared(ctypes.byref(ok), 3, one, one, blk, 3 * per_set - 1, None) == 3
    assert lib.dd_prepare_shared(ctypes.byref(ok), 3, one, one, None, 3 * per_set, None) == 3
    for fn in (lib.dd_fwd_shared, lib.dd_bwd_input_shared):
        assert fn(ctypes.byref(ok), 0, one, blk, 8 * per_set, one, None) == 1
        assert fn(ctypes.byref(ok), 9, one, blk, 9 * per_set, one, None) == 2
        assert fn(ctypes.byref(ok), 3, one, blk, 3 * per_set - 1, one, None) == 3   # a block for fewer sets
        assert fn(ctypes.byref(ok), 3, one, ctypes.c_void_p(520), 3 * per_set, one, None) == 3
        assert fn(ctypes.byref(ok), 3, None, blk, 3 * per_set, one, None) == 1
        assert fn(ctypes.byref(ok), 3, one, blk, 3 * per_set, None, None) == 1
        # shapes and types the matrix-core kernels do not cover
        for bad in (_layer(T=8, M=768, N=768, K=8, dtype=0), _layer(T=8, M=100, N=768, K=8, dtype=1)):
            assert fn(ctypes.byref(bad), 3, one, blk, 1 << 30, one, None) == 2
        # no tokens: nothing to do
        assert fn(ctypes.byref(_layer(T=0, M=768, N=768, K=8, dtype=1)), 3, None, blk, 3 * per_set, None, None) == 0
    bad = _layer(T=8, M=768, N=768, K=8, dtype=0)
    assert lib.dd_prepare_shared(ctypes.byref(bad), 3, one, one, blk, 1 << 30, None) == 2


def test_diagheur_rules(lib):
    one = ctypes.c_void_p(256)
    l = _layer(M=768, N=768, K=77)
    need = lib.dd_workspace_bytes(binding.DD_OP_DIAGHEUR, ctypes.byref(l), 0)
    assert need == 2 * 768 * 4 + 512  # scores, table, kept offsets; each part rounded up to 256 bytes
    args = (one, one, one, one, one, ctypes.c_void_p(512), need, None)
    assert lib.dd_diagheur_update(768, 77, -1, *args) == 1
    assert lib.dd_diagheur_update(768, 77, 78, *args) == 1           # more than are active
    assert lib.dd_diagheur_update(100, 77, 24, *args) == 1           # more than there are candidates to grow
    assert lib.dd_diagheur_update(768, 0, 0, *args) == 1
    assert lib.dd_diagheur_update(1 << 20, 77, 3, *args) == 2
    assert lib.dd_diagheur_update(768, 77, 7, None, one, one, one, one, ctypes.c_void_p(512), need, None) == 1
    assert lib.dd_diagheur_update(768, 77, 7, one, one, one, one, one, None, 0, None) == 3
    assert lib.dd_diagheur_update(768, 77, 7, one, one, one, one, one, ctypes.c_void_p(512), need - 1, None) == 3
    assert lib.dd_diag_magnitude(0, 8, 0, one, one, None) == 1
    assert lib.dd_diag_magnitude(4, 8, 5, one, one, None) == 1
    assert lib.dd_diag_magnitude(4, 8, 0, None, one, None) == 1


def test_binding_refuses_cpu_tensors():
    import torch
    X = torch.zeros(4, 8)
    off = torch.zeros(2, dtype=torch.int32)
    v = torch.zeros(2, 8)
    with pytest.raises(ValueError):
        dd.dd_fwd(X, off, v, 8)


def test_weight_gradient_workspace_covers_whichever_family_runs(lib):
    """Under DD_ALGO_AUTO the kernel family of dd_bwd_weight is settled at the call (X or dY not 16-byte aligned:
    vector kernels), and the families cut the tokens into different numbers of chunks; the size asked for must cover
    both.  A forced matrix-core call needs the matrix-core size only."""
    for T, M, N, K in ((25216, 768, 3072, 307), (50432, 768, 768, 77), (25216, 1024, 4096, 410), (300, 768, 768, 77)):
        sizes = {}
        for algo in (binding.DD_ALGO_AUTO, binding.DD_ALGO_VECTOR, binding.DD_ALGO_MATRIX, binding.DD_ALGO_PREPARED):
            l = _layer(T=T, M=M, N=N, K=K, dtype=1, algo=algo)
            sizes[algo] = lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT, ctypes.byref(l), 0)
        assert sizes[binding.DD_ALGO_AUTO] == max(sizes[binding.DD_ALGO_VECTOR], sizes[binding.DD_ALGO_MATRIX])
        assert sizes[binding.DD_ALGO_PREPARED] == sizes[binding.DD_ALGO_MATRIX] > 0


def test_few_diagonals_workspace_rules(lib):
    """The kernels for a handful of diagonals keep one block of partial sums per workgroup: at most 512 blocks and at
    most 16 MiB of them (64 blocks where one block alone is large).  DD_ALGO_VECTOR asks for them up to 16 diagonals,
    DD_ALGO_AUTO up to D / 192; the size covers the general vector kernels too (matrices that are not 16-byte aligned)."""
    def need(T, M, N, K, algo, dtype=1):
        l = _layer(T=T, M=M, N=N, K=K, dtype=dtype, algo=algo)
        return lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT, ctypes.byref(l), 0)
    V, A, X = binding.DD_ALGO_VECTOR, binding.DD_ALGO_AUTO, binding.DD_ALGO_MATRIX
    assert need(12608, 768, 768, 4, V) == 512 * 4 * 768 * 4
    assert need(12608, 768, 768, 16, V) == ((16 << 20) // (16 * 768 * 4)) * 16 * 768 * 4
    assert need(3000, 512, 4096, 16, V) == 512 * 16 * 512 * 4
    assert need(700, 1024, 4096, 16, V) == 256 * 16 * 1024 * 4
    assert need(700, 8192, 8192, 16, V) == 64 * 16 * 8192 * 4
    assert need(12608, 768, 768, 4, A) == max(need(12608, 768, 768, 4, V), need(12608, 768, 768, 4, X))
    # beyond D / 192 diagonals DD_ALGO_AUTO no longer counts on these kernels; beyond sixteen nobody does
    for K in (5, 17):
        plain_vector = need(12608, 768, 768, K, V) if K > 16 else None
        assert need(12608, 768, 768, K, A) >= need(12608, 768, 768, K, X)
        if plain_vector is not None:
            assert plain_vector < 512 * K * 768 * 4
    # fp32 storage and widths that are no multiple of 128 never take them
    assert need(12608, 768, 768, 4, V, dtype=0) < 512 * 4 * 768 * 4
    assert need(12608, 700, 700, 4, V) < 512 * 4 * 700 * 4


def test_batched_prepare_rules(lib):
    one, blk = ctypes.c_void_p(256), ctypes.c_void_p(512)
    ok = _layer(T=0, M=768, N=3072, K=30, dtype=1)
    per = lib.dd_workspace_bytes(binding.DD_OP_PREPARE, ctypes.byref(ok), 0)
    assert per % 256 == 0  # layer i's block starts where layer i-1's ends, and must be as aligned as a block of its own
    assert lib.dd_prepare_batched(ctypes.byref(ok), -1, one, one, blk, 12 * per, None) == 1
    assert lib.dd_prepare_batched(ctypes.byref(ok), 0, None, None, None, 0, None) == 0   # nothing to do
    assert lib.dd_prepare_batched(ctypes.byref(ok), 12, None, one, blk, 12 * per, None) == 1
    assert lib.dd_prepare_batched(ctypes.byref(ok), 12, one, None, blk, 12 * per, None) == 1
    assert lib.dd_prepare_batched(ctypes.byref(ok), 12, one, one, blk, 12 * per - 1, None) == 3
    assert lib.dd_prepare_batched(ctypes.byref(ok), 12, one, one, None, 12 * per, None) == 3
    assert lib.dd_prepare_batched(ctypes.byref(ok), 70000, one, one, blk, 1 << 62, None) == 2
    for bad in (_layer(M=768, N=768, K=8, dtype=0), _layer(M=100, N=768, K=8, dtype=1),
                _layer(M=768, N=768, K=8, dtype=1, algo=binding.DD_ALGO_VECTOR)):
        assert lib.dd_prepare_batched(ctypes.byref(bad), 3, one, one, blk, 1 << 30, None) == 2


def test_soft_path_folded_rules(lib):
    one, blk = ctypes.c_void_p(256), ctypes.c_void_p(512)
    f = ctypes.c_float
    assert lib.dd_select_soft(1, 8, 0, f(1.0), one, one, one, None) == 1
    assert lib.dd_select_soft(1, 8, 9, f(1.0), one, one, one, None) == 1
    assert lib.dd_select_soft(1, 8, 2, f(0.0), one, one, one, None) == 1      # temperature must be positive
    assert lib.dd_select_soft(1, 8, 2, f(float("nan")), one, one, one, None) == 1
    assert lib.dd_select_soft(1, 8, 2, f(1.0), None, one, one, None) == 1
    assert lib.dd_select_soft(1, 8, 2, f(1.0), one, None, one, None) == 1
    assert lib.dd_select_soft(1, 8, 2, f(1.0), one, one, None, None) == 1
    assert lib.dd_select_soft(1, 1 << 20, 2, f(1.0), one, one, one, None) == 2
    assert lib.dd_select_soft(0, 8, 2, f(1.0), None, None, None, None) == 0
    ok = _layer(T=100, M=768, N=768, K=30, dtype=1)
    need = lib.dd_workspace_bytes(binding.DD_OP_PREPARE, ctypes.byref(ok), 0)
    assert lib.dd_prepare_scaled(ctypes.byref(ok), None, one, one, blk, need, None) == 1
    assert lib.dd_prepare_scaled(ctypes.byref(ok), one, None, one, blk, need, None) == 1
    assert lib.dd_prepare_scaled(ctypes.byref(ok), one, one, None, blk, need, None) == 1
    assert lib.dd_prepare_scaled(ctypes.byref(ok), one, one, one, blk, need - 1, None) == 3
    assert lib.dd_prepare_scaled(ctypes.byref(_layer(M=768, N=768, K=8, dtype=0)), one, one, one, blk, need, None) == 2
    ws_need = lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT_SCALED, ctypes.byref(ok), 0)
    plain = lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT, ctypes.byref(_layer(T=100, M=768, N=768, K=30, dtype=1, algo=binding.DD_ALGO_MATRIX)), 0)
    assert ws_need > plain > 0  # the partial sums, then the dot products
    args = lambda **kw: [kw.get(k, one) for k in ("X", "dY", "off", "alpha", "V", "dV", "dalpha")]
    for missing in ("X", "dY", "off", "alpha", "V", "dV", "dalpha"):
        assert lib.dd_bwd_weight_scaled(ctypes.byref(ok), *args(**{missing: None}), blk, ws_need, None) == 1
    assert lib.dd_bwd_weight_scaled(ctypes.byref(ok), *args(), blk, ws_need - 1, None) == 3
    assert lib.dd_bwd_weight_scaled(ctypes.byref(ok), *args(), None, ws_need, None) == 3
    for bad in (_layer(T=8, M=768, N=768, K=8, dtype=0), _layer(T=8, M=100, N=768, K=8, dtype=1),
                _layer(T=8, M=768, N=768, K=8, dtype=1, algo=binding.DD_ALGO_VECTOR)):
        assert lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT_SCALED, ctypes.byref(bad), 0) == 0
        assert lib.dd_bwd_weight_scaled(ctypes.byref(bad), *args(), blk, 1 << 30, None) == 2
    assert lib.dd_bwd_weight_scaled(ctypes.byref(_layer(T=0, M=768, N=768, K=8, dtype=1)), *args(), blk, 1 << 30, None) == 1
    # X that starts at an odd element: the matrix-core kernels need 16-byte alignment
    assert lib.dd_bwd_weight_scaled(ctypes.byref(ok), *args(X=ctypes.c_void_p(258)), blk, ws_need, None) == 2


def test_backward_as_one_call_rules(lib):
    one, blk = ctypes.c_void_p(256), ctypes.c_void_p(512)
    ok = _layer(T=100, M=768, N=3072, K=30, dtype=1)
    need = lib.dd_workspace_bytes(binding.DD_OP_BWD, ctypes.byref(ok), 0)
    a = lib.dd_workspace_bytes(binding.DD_OP_BWD_INPUT, ctypes.byref(ok), 0)
    b = lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT, ctypes.byref(ok), 0)
    assert need == max(a, b)  # the two products take their scratch from one block, one after the other
    prep = _layer(T=100, M=768, N=3072, K=30, dtype=1, algo=binding.DD_ALGO_PREPARED)
    forced = _layer(T=100, M=768, N=3072, K=30, dtype=1, algo=binding.DD_ALGO_MATRIX)
    assert lib.dd_workspace_bytes(binding.DD_OP_BWD, ctypes.byref(prep), 0) == lib.dd_workspace_bytes(
        binding.DD_OP_BWD_WEIGHT, ctypes.byref(forced), 0)
    pb = lib.dd_workspace_bytes(binding.DD_OP_PREPARE, ctypes.byref(prep), 0)
    # (layer, X, dY, offsets, values, prepared, prepared_bytes, dX, dValues, ws, ws_bytes, stream)
    assert lib.dd_bwd(ctypes.byref(ok), one, one, one, one, None, 0, one, one, blk, need - 1, None) == 3
    assert lib.dd_bwd(ctypes.byref(ok), one, one, one, one, None, 0, one, one, None, need, None) == 3
    assert lib.dd_bwd(ctypes.byref(ok), one, one, None, one, None, 0, one, one, blk, need, None) == 1
    assert lib.dd_bwd(ctypes.byref(ok), one, one, one, None, None, 0, one, one, blk, need, None) == 1
    assert lib.dd_bwd(ctypes.byref(ok), one, None, one, one, None, 0, one, one, blk, need, None) == 1
    assert lib.dd_bwd(ctypes.byref(ok), one, one, one, one, None, 0, None, one, blk, need, None) == 1
    assert lib.dd_bwd(ctypes.byref(prep), one, one, one, None, None, pb, one, one, blk, need, None) == 1   # no block
    assert lib.dd_bwd(ctypes.byref(prep), one, one, one, None, blk, pb - 1, one, one, blk, need, None) == 3
    blocks = _layer(T=100, M=768, N=3072, K=30, dtype=1, algo=binding.DD_ALGO_BLOCKS)
    assert lib.dd_workspace_bytes(binding.DD_OP_BWD, ctypes.byref(blocks), 0) == 0
    assert lib.dd_bwd(ctypes.byref(blocks), one, one, one, one, blk, pb, one, one, blk, need, None) == 2


def test_block_skipping_rules(lib):
    one, blk = ctypes.c_void_p(256), ctypes.c_void_p(512)
    l = _layer(T=64, M=768, N=768, K=77, dtype=1, algo=binding.DD_ALGO_BLOCKS)
    need = lib.dd_workspace_bytes(binding.DD_OP_FWD, ctypes.byref(l), 0)
    assert need == 2 * 768 * 768 * 2 == lib.dd_workspace_bytes(binding.DD_OP_BWD_INPUT, ctypes.byref(l), 0)
    for fn in (lib.dd_fwd, lib.dd_bwd_input):
        assert fn(ctypes.byref(l), one, None, None, one, blk, need, None) == 1       # the offsets are read
        assert fn(ctypes.byref(l), one, one, None, one, blk, need - 1, None) == 3
        assert fn(ctypes.byref(l), one, one, None, one, None, need, None) == 3
        assert fn(ctypes.byref(_layer(T=64, M=768, N=768, K=77, dtype=0, algo=binding.DD_ALGO_BLOCKS)), one, one, None, one, blk, need, None) == 2
        assert fn(ctypes.byref(_layer(T=64, M=100, N=768, K=7, dtype=1, algo=binding.DD_ALGO_BLOCKS)), one, one, None, one, blk, 1 << 30, None) == 2
        assert fn(ctypes.byref(_layer(T=64, M=16384, N=128, K=7, dtype=1, algo=binding.DD_ALGO_BLOCKS)), one, one, None, one, blk, 1 << 30, None) == 2
        assert fn(ctypes.byref(_layer(T=0, M=768, N=768, K=77, dtype=1, algo=binding.DD_ALGO_BLOCKS)), None, one, None, None, blk, need, None) == 0


def test_static_scratch_rules(lib):
    one = ctypes.c_void_p(256)
    assert lib.dd_static_scratch_bytes() == 32 << 20
    big = _layer(T=25216, M=1024, N=4096, K=819, dtype=1)
    assert lib.dd_workspace_bytes(binding.DD_OP_BWD_WEIGHT, ctypes.byref(big), 0) > 32 << 20
    assert lib.dd_bwd_weight_static(ctypes.byref(big), one, one, one, one, None) == 3      # before any launch or lookup
    assert lib.dd_bwd_weight_static(ctypes.byref(_layer(K=0)), one, one, one, one, None) == 1
