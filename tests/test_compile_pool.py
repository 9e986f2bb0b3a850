"""The pool of compile workers: the limit on the time one instantiation may take (no GPU).

Runs in a process of its own: the pool is one per process and the other tests share theirs."""
import os
import subprocess
import sys
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SCRIPT = textwrap.dedent("""
    import sys
    sys.path.insert(0, %r)
    import paper_2006_05664_amd as P
    assert P.opevo_compile_pool_start(6) == 6
    op = P.opevo_op_create(P.OPEVO_MATMUL, (512, 1024, 1024), P.OPEVO_BF16)
    cfgs = [[2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1], [2, 2, 2, 64, 8, 2, 2, 32, 32, 32, 1], [2, 2, 2, 64, 8, 2, 2, 32, 64, 16, 1],
            [4, 2, 1, 64, 8, 2, 2, 32, 16, 64, 1]]
    # no compilation ends within 10 ms: the caller is answered that the member cannot be evaluated, the workers
    # finish in the background and return to the pool
    P.opevo_compile_pool_deadline(0.01)
    for i in range(3):
        try:
            P.opevo_kernel_build(op, P.OPEVO_TILE4, cfgs[i])
            raise SystemExit("member %%d was built within 10 ms?" %% i)
        except P.OpevoError as e:
            assert e.status == P.OPEVO_E_INVALID and "deadline" in e.message, (e.status, e.message)
    assert P.opevo_compile_pool_start(6) == 6              # idempotent: answers the workers alive; none was ended
    # no limit again: a member that was refused is built now (nothing of the failed attempt was cached), and so
    # are more members than there are workers at once (every worker is back once its late compilation has ended)
    P.opevo_compile_pool_deadline(0.0)
    from concurrent.futures import ThreadPoolExecutor
    more = [[2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1], [4, 2, 1, 64, 8, 2, 2, 32, 16, 64, 1], [2, 4, 1, 64, 8, 2, 2, 32, 16, 64, 1],
            [2, 2, 2, 64, 16, 2, 1, 32, 16, 64, 1], [2, 2, 2, 64, 4, 2, 4, 32, 16, 64, 1], [1, 4, 2, 64, 8, 2, 2, 32, 16, 64, 1],
            [2, 2, 2, 64, 8, 2, 2, 32, 8, 128, 1], [2, 2, 2, 64, 8, 2, 2, 32, 4, 256, 0]]
    with ThreadPoolExecutor(8) as ex:
        for k, ms in ex.map(lambda c: P.opevo_kernel_build(op, P.OPEVO_TILE4, c), more):
            assert P.opevo_kernel_code_size(k) > 0
            P.opevo_kernel_destroy(k)
    try:
        P.opevo_compile_pool_deadline(-1.0)
        raise SystemExit("a negative limit was accepted")
    except P.OpevoError as e:
        assert e.status == P.OPEVO_E_ARG
    P.opevo_op_destroy(op)
    P.opevo_compile_pool_stop()
    print("ok")
""") % ROOT


def test_a_compilation_that_overruns_is_not_waited_for_and_counts_as_invalid():
    r = subprocess.run([sys.executable, "-c", SCRIPT], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.stdout[-2000:], r.stderr[-2000:])
