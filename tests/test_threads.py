"""Host threads and the boundary: options, the lent workspace, the record of the last launch and the
planner's cache are per host thread, so two threads that plan (or launch) different problems at the
same time each read back their own answer.  CPU only: the plans are dry runs."""
import ctypes
import threading

from paper_2604_23798_amd import elsa

P = ctypes.c_void_p(1 << 20)          # 256-byte aligned, never dereferenced in a dry run


def _worker(kind, rounds, errors, barrier):
    lib = elsa.raw()
    try:
        assert elsa.elsa_get_option(elsa.OPT_DRY_RUN) == 0           # a new thread starts from the defaults
        elsa.elsa_set_option(elsa.OPT_DRY_RUN, 1)
        barrier.wait()
        for i in range(rounds):
            if kind == 0:
                # headline shape, forced 256-row tile, no workspace
                elsa.elsa_set_option(elsa.OPT_VARIANT, 2)
                rc = lib.elsa_attn_fwd(P, P, P, P, 1, 16, 16384, 64, 0.125, 0, 0, None)
                want = ("mfma_q256_w4", 1)
            elif kind == 1:
                # decoding against 32K keys with a workspace of this thread's own: 16 chunks
                assert lib.elsa_set_workspace(P, 256 << 20) == 0
                rc = lib.elsa_attn_fwd_cross(P, P, P, P, None, 2, 40, 1, 32768, 128, 0.088, 1, None, 0, None)
                want = ("fma_decode_q1", 16)
            else:
                # FP16 small causal problem: 64-row tile, alternating with a second shape so that the
                # planner's one-entry cache is exercised
                n = 2048 if i % 2 == 0 else 4096
                rc = lib.elsa_attn_fwd(P, P, P, P, 1, 16, n, 64, 0.125, 1, 1, None)
                want = (("mfma16_q64_xw2", "mfma16_xwave") if n == 2048 else ("mfma16_q64_xw2",), 1)
            assert rc == 0
            got = (elsa.elsa_last_kernel(), elsa.elsa_last_splits())
            ok = got[1] == want[1] and (got[0] in want[0] if isinstance(want[0], tuple) else got[0] == want[0])
            assert ok, (kind, i, got, want)
    except BaseException as e:       # noqa: BLE001  (reported by the main thread)
        errors.append((kind, repr(e)))
        try:
            barrier.abort()
        except Exception:
            pass


def test_concurrent_plans_do_not_see_each_other():
    errors = []
    n_threads = 6
    barrier = threading.Barrier(n_threads)
    ts = [threading.Thread(target=_worker, args=(i % 3, 300, errors, barrier)) for i in range(n_threads)]
    for t in ts:
        t.start()
    for t in ts:
        t.join(120)
    assert not errors, errors
    # nothing leaked into the main thread
    assert elsa.elsa_get_option(elsa.OPT_DRY_RUN) == 0 and elsa.elsa_get_option(elsa.OPT_VARIANT) == 0
