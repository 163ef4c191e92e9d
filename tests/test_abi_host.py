"""Host-only checks of the C ABI: the library loads, exports every declared
symbol, its structs match the header as a C compiler lays them out, and
argument validation returns the documented codes before anything is enqueued
(no GPU is touched)."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nadmm.h")

from paper_1807_07132_amd import nadmm  # noqa: E402


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(nadmm.LIB_PATH):
        from paper_1807_07132_amd import build
        build.build(verbose=False)
    return nadmm.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nadmm_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"nadmm_loss_grad", "nadmm_hessvec", "nadmm_cg_solve", "nadmm_line_search", "nadmm_local_newton",
            "nadmm_workspace_bytes"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert lib.nadmm_version() >= 100
    assert lib.nadmm_status_string(0) == b"ok"
    assert b"workspace" in lib.nadmm_status_string(nadmm.NADMM_EWORKSPACE)


def test_struct_layout_matches_the_header(tmp_path):
    src = tmp_path / "sizes.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "nadmm.h"\n'
        "int main(void){printf(\"%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\\n\", sizeof(nadmm_problem), sizeof(nadmm_params),"
        " sizeof(nadmm_stats), offsetof(nadmm_problem, d_labels), offsetof(nadmm_problem, d_z),"
        " offsetof(nadmm_stats, loss_initial), offsetof(nadmm_stats, grad_norm), sizeof(nadmm_admm_params),"
        " sizeof(nadmm_admm_stats), offsetof(nadmm_admm_params, local), offsetof(nadmm_admm_stats, d_trace),"
        " offsetof(nadmm_problem, sparse), sizeof(nadmm_sparse), offsetof(nadmm_sparse, d_val_t),"
        " offsetof(nadmm_admm_params, rb_tau), offsetof(nadmm_admm_stats, rho_scale_trace));return 0;}\n")
    exe = tmp_path / "sizes"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", f"-I{os.path.join(ROOT, 'include')}", str(src), "-o", str(exe)])
    got = [int(v) for v in subprocess.check_output([str(exe)]).split()]
    want = [C.sizeof(nadmm.nadmm_problem), C.sizeof(nadmm.nadmm_params), C.sizeof(nadmm.nadmm_stats),
            nadmm.nadmm_problem.d_labels.offset, nadmm.nadmm_problem.d_z.offset,
            nadmm.nadmm_stats.loss_initial.offset, nadmm.nadmm_stats.grad_norm.offset,
            C.sizeof(nadmm.nadmm_admm_params), C.sizeof(nadmm.nadmm_admm_stats), nadmm.nadmm_admm_params.local.offset,
            nadmm.nadmm_admm_stats.d_trace.offset, nadmm.nadmm_problem.sparse.offset, C.sizeof(nadmm.nadmm_sparse),
            nadmm.nadmm_sparse.d_val_t.offset, nadmm.nadmm_admm_params.rb_tau.offset,
            nadmm.nadmm_admm_stats.rho_scale_trace.offset]
    assert got == want


def fake_problem(n=1000, p=20, Cc=3, lda=None, rho=1.0, lam=1e-3, A=0x1000, labels=0x2000):
    return nadmm.nadmm_problem(A, n, p, p if lda is None else lda, labels, Cc, 1.0, lam, rho, None, None, None)


def fake_sparse(nnz=5000, **kw):
    f = dict(nnz=nnz, d_row_ptr=0x4000, d_col_idx=0x5000, d_val=0x6000, d_col_ptr=0x7000, d_row_idx=0x8000,
             d_val_t=0x9000)
    f.update(kw)
    return nadmm.nadmm_sparse(f["nnz"], f["d_row_ptr"], f["d_col_idx"], f["d_val"], f["d_col_ptr"], f["d_row_idx"],
                              f["d_val_t"])


def sparse_problem(sp, **kw):
    prob = fake_problem(A=None, **kw)
    prob.sparse = C.pointer(sp)
    return prob


def test_sparse_problems_on_the_host(lib):
    fake = C.c_void_p(0x3000)
    sp = fake_sparse()
    prob = sparse_problem(sp, n=1000, p=3000, Cc=5)
    need = lib.nadmm_workspace_bytes(C.byref(prob), None)
    assert need > 0 and need % 256 == 0
    assert lib.nadmm_query_kernel_path(C.byref(prob)) == 5
    # no dense array is needed, and a dense problem never takes the sparse path
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem())) in (1, 2, 3, 4)
    prev = lib.nadmm_set_kernel_path(5)
    try:
        assert lib.nadmm_query_kernel_path(C.byref(fake_problem())) == nadmm.NADMM_EUNSUPPORTED
        assert lib.nadmm_query_kernel_path(C.byref(prob)) == 5
        lib.nadmm_set_kernel_path(1)
        assert lib.nadmm_query_kernel_path(C.byref(prob)) == nadmm.NADMM_EUNSUPPORTED
    finally:
        lib.nadmm_set_kernel_path(prev)
    # more stored entries need more windows, hence more workspace
    sp_big = fake_sparse(nnz=50_000_000)
    assert lib.nadmm_workspace_bytes(C.byref(sparse_problem(sp_big, n=1000, p=3000, Cc=5)), None) > need
    for bad in (fake_sparse(nnz=-1), fake_sparse(d_row_ptr=None), fake_sparse(d_col_ptr=None), fake_sparse(d_val=None),
                fake_sparse(d_row_idx=None), fake_sparse(d_val_t=None), fake_sparse(d_col_idx=None)):
        pb = sparse_problem(bad, n=1000, p=3000, Cc=5)
        assert lib.nadmm_workspace_bytes(C.byref(pb), None) == 0
        assert lib.nadmm_hessvec(C.byref(pb), fake, fake, fake, fake, 1 << 30, None) == nadmm.NADMM_EINVAL
    # an empty matrix needs no index or value arrays
    empty = fake_sparse(nnz=0, d_col_idx=None, d_val=None, d_row_idx=None, d_val_t=None)
    assert lib.nadmm_workspace_bytes(C.byref(sparse_problem(empty, n=1000, p=3000, Cc=5)), None) > 0
    huge = sparse_problem(sp, n=(1 << 31), p=30, Cc=3)
    assert lib.nadmm_hessvec(C.byref(huge), fake, fake, fake, fake, 1 << 30, None) == nadmm.NADMM_EUNSUPPORTED
    assert lib.nadmm_hessvec(C.byref(prob), fake, fake, fake, fake, need - 1, None) == nadmm.NADMM_EWORKSPACE


def test_workspace_bytes(lib):
    small = lib.nadmm_workspace_bytes(C.byref(fake_problem()), None)
    big = lib.nadmm_workspace_bytes(C.byref(fake_problem(n=60000, p=784, Cc=10)), None)
    assert small > 0 and big > small and small % 256 == 0
    assert big >= 4 * 60000 * 9 * 4                      # four n x (C-1) row buffers
    assert big < 1 << 30
    assert lib.nadmm_workspace_bytes(C.byref(fake_problem(n=0)), None) == 0
    assert lib.nadmm_workspace_bytes(None, None) == 0


def test_workspace_bytes_with_parameters(lib):
    """With parameters the size may add the history of directional logits (max_cg arrays of n (C-1) floats) where the
    single-pass matrix-core path applies and the history is cheaper than the pass over A it replaces."""
    rows = 60000 * 9 * 4
    head = fake_problem(n=60000, p=784, Cc=10)
    base = lib.nadmm_workspace_bytes(C.byref(head), None)
    for max_cg, kept in ((10, True), (29, True), (30, False), (0, False), (33, False)):   # 3 max_cg (C-1) <= p, max_cg <= 32
        pr = nadmm.make_params(10, max_cg, 10, 0.0, 0.0, 1e-4, 0.5)
        need = lib.nadmm_workspace_bytes(C.byref(head), C.byref(pr))
        assert need % 256 == 0
        if kept:
            assert max_cg * rows <= need - base < max_cg * (rows + 256)
        else:
            assert need == base
    pr = nadmm.make_params(10, 10, 10, 0.0, 0.0, 1e-4, 0.5)
    for other in (fake_problem(n=1375000, p=28, Cc=2),            # thin-data path
                  fake_problem(n=50000, p=3072, Cc=10),           # column-sliced path
                  fake_problem(n=50000, p=3072, Cc=10, lda=3073)):  # the same on rows that are not 16-byte aligned
        assert lib.nadmm_workspace_bytes(C.byref(other), C.byref(pr)) == lib.nadmm_workspace_bytes(C.byref(other), None)


@pytest.mark.parametrize("kw,code", [
    (dict(n=0), nadmm.NADMM_EINVAL),
    (dict(p=0), nadmm.NADMM_EINVAL),
    (dict(Cc=1), nadmm.NADMM_EINVAL),
    (dict(lda=19), nadmm.NADMM_EINVAL),
    (dict(rho=0.0), nadmm.NADMM_EINVAL),
    (dict(rho=float("nan")), nadmm.NADMM_EINVAL),
    (dict(lam=-1.0), nadmm.NADMM_EINVAL),
    (dict(A=None), nadmm.NADMM_EINVAL),
    (dict(Cc=40), nadmm.NADMM_EUNSUPPORTED),
])
def test_invalid_problems_are_rejected_on_the_host(lib, kw, code):
    prob = fake_problem(**kw)
    fake = C.c_void_p(0x3000)
    assert lib.nadmm_hessvec(C.byref(prob), fake, fake, fake, fake, 1 << 30, None) == code
    assert lib.nadmm_loss_grad(C.byref(prob), fake, fake, fake, fake, 1 << 30, None) == code
    params = nadmm.make_params()
    assert lib.nadmm_local_newton(C.byref(prob), fake, C.byref(params), None, fake, 1 << 30, None) == code


def test_null_arguments_and_workspace_errors(lib):
    prob = fake_problem()
    fake = C.c_void_p(0x3000)
    need = lib.nadmm_workspace_bytes(C.byref(prob), None)
    assert lib.nadmm_hessvec(C.byref(prob), None, fake, fake, fake, need, None) == nadmm.NADMM_EINVAL
    assert lib.nadmm_hessvec(C.byref(prob), fake, fake, None, fake, need, None) == nadmm.NADMM_EINVAL
    assert lib.nadmm_hessvec(C.byref(prob), fake, fake, fake, None, need, None) == nadmm.NADMM_EWORKSPACE
    assert lib.nadmm_hessvec(C.byref(prob), fake, fake, fake, fake, need - 1, None) == nadmm.NADMM_EWORKSPACE
    assert lib.nadmm_hessvec(C.byref(prob), fake, fake, fake, C.c_void_p(0x3010), need, None) == nadmm.NADMM_EWORKSPACE
    # labels are required by the objective but not by the Hessian-vector product
    nolab = fake_problem(labels=None)
    assert lib.nadmm_loss_grad(C.byref(nolab), fake, fake, fake, fake, need, None) == nadmm.NADMM_EINVAL
    assert lib.nadmm_cg_solve(C.byref(prob), fake, fake, fake, -1, 0.0, None, None, fake, need, None) == nadmm.NADMM_EINVAL
    assert lib.nadmm_cg_solve(C.byref(prob), fake, None, fake, 5, 0.0, None, None, fake, need, None) == nadmm.NADMM_EINVAL


@pytest.mark.parametrize("beta,gamma,max_ls,code", [
    (0.0, 0.5, 10, nadmm.NADMM_EINVAL), (1.0, 0.5, 10, nadmm.NADMM_EINVAL),
    (1e-4, 0.0, 10, nadmm.NADMM_EINVAL), (1e-4, 1.0, 10, nadmm.NADMM_EINVAL),
    (1e-4, 0.5, -1, nadmm.NADMM_EINVAL), (1e-4, 0.5, 63, nadmm.NADMM_EUNSUPPORTED),
])
def test_line_search_parameters_are_validated(lib, beta, gamma, max_ls, code):
    prob = fake_problem()
    fake = C.c_void_p(0x3000)
    need = lib.nadmm_workspace_bytes(C.byref(prob), None)
    rc = lib.nadmm_line_search(C.byref(prob), fake, fake, fake, 1.0, beta, gamma, max_ls, fake, fake, fake, fake, need, None)
    assert rc == code
    params = nadmm.make_params(armijo_beta=beta, backtrack_gamma=gamma, max_ls=max_ls)
    assert lib.nadmm_local_newton(C.byref(prob), fake, C.byref(params), None, fake, need, None) == code


def test_kernel_path_switch(lib):
    prev = lib.nadmm_set_kernel_path(1)
    assert prev in (0, 1, 2, 3, 4)
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem())) == 1
    assert lib.nadmm_set_kernel_path(7) == nadmm.NADMM_EINVAL
    lib.nadmm_set_kernel_path(0)
    # automatic selection: thin data -> 3, medium width -> 2, wide or many classes -> 4; rows that are not 16-byte aligned
    # take the same from 48 columns on, the vector kernels (1) below that
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=1000, p=20, Cc=3))) == 3
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=60000, p=784, Cc=10))) == 2
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=50000, p=3072, Cc=10))) == 4
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=250000, p=2000, Cc=20))) == 4
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=45, Cc=5))) == 1
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=49, Cc=5))) == 2
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=48, Cc=5, A=0x1004))) == 2      # 4-byte aligned A
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=36, Cc=5))) == 2                 # aligned rows: any p
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=2001, Cc=5))) == 4               # wide and unaligned
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=49, Cc=20))) == 4                # many classes and unaligned
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=45, Cc=20))) == 1
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=49, Cc=20, A=0x1002))) == 1      # A not 4-byte aligned
    # forced: the any-stride variants take narrow rows too, down to one 16-byte piece
    lib.nadmm_set_kernel_path(2)
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=45, Cc=5))) == 2
    assert lib.nadmm_query_kernel_path(C.byref(fake_problem(n=500, p=3, Cc=5))) == nadmm.NADMM_EUNSUPPORTED
    lib.nadmm_set_kernel_path(0)
    # a forced path that cannot take the shape is reported, on the host
    lib.nadmm_set_kernel_path(3)
    fake = C.c_void_p(0x3000)
    wide = fake_problem(n=60000, p=784, Cc=10)
    need = lib.nadmm_workspace_bytes(C.byref(wide), None)
    assert lib.nadmm_hessvec(C.byref(wide), fake, fake, fake, fake, need, None) == nadmm.NADMM_EUNSUPPORTED
    lib.nadmm_set_kernel_path(prev)


def test_static_scratch_entry_point_validates_on_the_host(lib):
    """nadmm_hessvec_static rejects invalid arguments and problems beyond its built-in buffer before any device call."""
    fake = C.c_void_p(0x3000)
    cap = lib.nadmm_static_scratch_bytes()
    assert cap == 32 << 20
    head = fake_problem(n=60000, p=784, Cc=10)
    assert 0 < lib.nadmm_hessvec_static_bytes(C.byref(head)) < 20 << 20           # the headline shape fits
    assert lib.nadmm_hessvec_static_bytes(C.byref(head)) < lib.nadmm_workspace_bytes(C.byref(head), None)
    assert lib.nadmm_hessvec_static(C.byref(head), None, fake, fake, None) == nadmm.NADMM_EINVAL
    assert lib.nadmm_hessvec_static(C.byref(head), fake, fake, None, None) == nadmm.NADMM_EINVAL
    big = fake_problem(n=500000, p=2000, Cc=20)                                     # 49 MB of scratch
    assert lib.nadmm_hessvec_static_bytes(C.byref(big)) > cap
    assert lib.nadmm_hessvec_static(C.byref(big), fake, fake, fake, None) == nadmm.NADMM_ESCRATCH
    assert b"built-in" in lib.nadmm_status_string(nadmm.NADMM_ESCRATCH)
    bad = fake_problem(n=0, p=784, Cc=10)
    assert lib.nadmm_hessvec_static_bytes(C.byref(bad)) == 0
    assert lib.nadmm_hessvec_static(C.byref(bad), fake, fake, fake, None) == nadmm.NADMM_EINVAL


def test_product_path_does_not_import_the_oracle():
    code = ("import sys; sys.path.insert(0, %r); import paper_1807_07132_amd.nadmm, paper_1807_07132_amd.workloads;"
            "assert not any(m == 'oracle' or m.startswith('oracle.') for m in sys.modules)" % ROOT)
    subprocess.check_call([sys.executable, "-c", code])


def test_admm_host_validation(lib):
    params = nadmm.make_admm_params(3, nadmm.make_params(2, 5, 10))
    fake = C.c_void_p(0x4000)
    workers = (nadmm.nadmm_problem * 3)(*[fake_problem(n=500 + 10 * i) for i in range(3)])
    need = lib.nadmm_admm_workspace_bytes(workers, 3, C.byref(params))
    single = max(lib.nadmm_workspace_bytes(C.byref(workers[i]), None) for i in range(3))
    assert need > single
    assert lib.nadmm_admm_workspace_bytes(workers, 0, C.byref(params)) == 0
    assert lib.nadmm_admm_workspace_bytes(workers, nadmm.NADMM_MAX_WORKERS + 1, C.byref(params)) == 0
    call = lambda w, N, lam, prm, ws: lib.nadmm_admm_solve(w, N, lam, fake, fake, fake, C.byref(prm), None, fake, ws, None)
    assert call(workers, 3, 0.1, params, need - 1) == nadmm.NADMM_EWORKSPACE
    assert call(workers, 3, -0.1, params, need) == nadmm.NADMM_EINVAL
    bad = nadmm.make_admm_params(-1, nadmm.make_params(2, 5, 10))
    assert call(workers, 3, 0.1, bad, need) == nadmm.NADMM_EINVAL
    for kw in (dict(penalty_rule=2), dict(penalty_rule=1, rb_mu=0.5), dict(penalty_rule=1, rb_tau=1.0),
               dict(penalty_rule=1, rb_tau=float("nan"))):
        assert call(workers, 3, 0.1, nadmm.make_admm_params(3, nadmm.make_params(2, 5, 10), **kw), need) == nadmm.NADMM_EINVAL
    mixed = (nadmm.nadmm_problem * 2)(fake_problem(p=20), fake_problem(p=24))     # shards must agree in p and C
    assert lib.nadmm_admm_workspace_bytes(mixed, 2, C.byref(params)) == 0
    rho = (C.c_float * 2)(1.0, -1.0)
    assert lib.nadmm_admm_consensus(2, 40, fake, fake, fake, rho, 0.1, 0.0, 0.0, None, fake, 1 << 16, None) == nadmm.NADMM_EINVAL
    rho = (C.c_float * 2)(1.0, 1.0)
    assert lib.nadmm_admm_consensus(2, 40, fake, fake, fake, rho, 0.1, 0.0, 0.0, None, fake, 16, None) == nadmm.NADMM_EWORKSPACE


def test_kernel_path_switch_is_per_thread(lib):
    """The forced kernel path belongs to the calling host thread: another thread still sees the automatic choice."""
    import threading
    assert lib.nadmm_set_kernel_path(2) == 0
    try:
        seen = []
        t = threading.Thread(target=lambda: seen.append(lib.nadmm_set_kernel_path(1)))
        t.start()
        t.join()
        assert seen == [0]                                # the other thread's previous value: untouched by this one
        assert lib.nadmm_set_kernel_path(2) == 2          # and its own setting did not reach this thread
    finally:
        lib.nadmm_set_kernel_path(0)
