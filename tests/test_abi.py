"""Host-side checks that need no GPU: the library loads, exports what the header declares,
the schedule entry points agree bit for bit with the oracle's generator, argument errors."""
import os
import re

import pytest

import paper_1806_03377_amd as pd
from oracle.schedule import schedule_1f1b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            src = open(os.path.join(ROOT, "include", fn)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names |= set(re.findall(r"\b(pd_[a-z0-9_]+)\s*\(", src))
    return names


def test_every_declared_symbol_is_exported():
    import ctypes
    lib = ctypes.CDLL(pd.binding.LIB_PATH)
    decl = _declared()
    assert {"pd_stage_create", "pd_forward", "pd_backward", "pd_update", "pd_schedule_1f1b"} <= decl
    for name in sorted(decl):
        assert hasattr(lib, name), name
    assert decl == set(pd.binding.EXPORTED)


@pytest.mark.parametrize("S", range(1, 7))
def test_schedule_matches_oracle_bit_exact(S):
    for noam in range(1, S + 1):
        for M in (0, 1, 2, 3, 5, 8, 3 * S, 64):
            for s in range(S):
                got = pd.pd_schedule_1f1b(S, noam, M, s)
                ref = [tuple(o) for o in schedule_1f1b(S, noam, M, s)] if M else []
                assert got == ref, (S, noam, M, s)


@pytest.mark.parametrize("S", range(1, 6))
def test_vertical_sync_schedule_matches_oracle_bit_exact(S):
    for noam in range(1, S + 1):
        for M in (0, 1, 2, 5, 3 * S, 40):
            for s in range(S):
                got = pd.pd_schedule_1f1b_vertical_sync(S, noam, M, s)
                ref = [tuple(o) for o in schedule_1f1b(S, noam, M, s, vertical_sync=True)] if M else []
                assert got == ref, (S, noam, M, s)
    with pytest.raises(pd.PdError):
        pd.pd_schedule_1f1b_vertical_sync(3, 3, 4, 3)


def test_schedule_with_forced_depth():
    for depth in (1, 2, 4, 7):
        for M in (1, 3, 4, 9, 20):
            got = pd.pd_schedule_1f1b_depth(depth, M)
            ref = [tuple(o) for o in schedule_1f1b(1, 1, M, 0, depth_override=depth)]
            assert got == ref


def test_schedule_argument_errors():
    with pytest.raises(pd.PdError) as e:
        pd.pd_schedule_1f1b(4, 4, 8, 4)
    assert e.value.status == pd.PD_EINVAL and "schedule" in str(e.value)
    with pytest.raises(pd.PdError):
        pd.pd_schedule_1f1b(0, 1, 8, 0)
    with pytest.raises(pd.PdError):
        pd.pd_schedule_1f1b_depth(0, 8)
    # capacity too small -> PD_ENOMEM, count still reported
    import ctypes as C
    arr = (pd.binding.pd_op * 2)()
    n = C.c_size_t(0)
    rc = pd.binding._lib.pd_schedule_1f1b(4, 4, 8, 0, arr, 2, C.byref(n))
    assert rc == pd.PD_ENOMEM and n.value == 24


def test_query_bytes_and_config_errors():
    import pd_inputs as gen
    cfg = pd.make_config(gen.config2_vgg_fc(), in_flight_override=4, minibatch=64, precision=pd.PD_BF16_F32ACC)
    n = pd.pd_stage_query_bytes(cfg)
    P = 123642856
    # ring of 4 bf16 copies + fp32 staging area for the master weights + fp32 momentum + the 16-bit remainders that,
    # with the latest ring copy, ARE the master weights of Linear layers dominate
    assert 4 * 2 * P + 8 * P + 2 * P <= n < 4 * 2 * P + 8 * P + 2 * P + 200 * 2 ** 20
    bad = pd.make_config([("linear", 30, 20, True)], minibatch=4, precision=pd.PD_BF16_F32ACC)
    with pytest.raises(pd.PdError) as e:
        pd.pd_stage_query_bytes(bad)
    assert e.value.status == pd.PD_EINVAL and "divisible by 8" in str(e.value)
    bad = pd.make_config([("linear", 32, 16, False), ("linear", 8, 8, False)], minibatch=4)
    with pytest.raises(pd.PdError):
        pd.pd_stage_query_bytes(bad)
    bad = pd.make_config([("softmax_xent", 8)], minibatch=4)
    with pytest.raises(pd.PdError):
        pd.pd_stage_query_bytes(bad)
    bad = pd.make_config([("linear", 8, 8, False)], minibatch=4, stage_index=2, num_stages=2)
    with pytest.raises(pd.PdError):
        pd.pd_stage_query_bytes(bad)
    bad = pd.make_config([("linear", 8, 8, False)], minibatch=4, optimizer=7)
    with pytest.raises(pd.PdError) as e:
        pd.pd_stage_query_bytes(bad)
    assert e.value.status == pd.PD_EINVAL and "optimizer" in str(e.value)
    bad = pd.make_config([("linear", 8, 8, False)], minibatch=4, optimizer=pd.PD_OPT_RMSPROP, eps=0.0)
    with pytest.raises(pd.PdError) as e:
        pd.pd_stage_query_bytes(bad)
    assert e.value.status == pd.PD_EINVAL and "eps" in str(e.value)
    ok = pd.make_config([("linear", 8, 8, False)], minibatch=4, optimizer=pd.PD_OPT_RMSPROP, eps=1.0)
    assert pd.pd_stage_query_bytes(ok) > 0


def test_replica_routing_and_config():
    assert [pd.pd_replica_route(i, 3) for i in range(7)] == [(0, 0), (1, 0), (2, 0), (0, 1), (1, 1), (2, 1), (0, 2)]
    for bad in ((-1, 2), (3, 0)):
        with pytest.raises(pd.PdError) as e:
            pd.pd_replica_route(*bad)
        assert e.value.status == pd.PD_EINVAL
    layers = [("linear", 64, 32, True), ("linear", 32, 16, False)]
    one = pd.pd_stage_query_bytes(pd.make_config(layers, minibatch=8, in_flight_override=2))
    cfg = pd.make_config(layers, minibatch=8, in_flight_override=2, replicas=2)
    first, more = pd.pd_stage_query_bytes(cfg), pd.pd_stage_replica_query_bytes(cfg)
    n_par = 64 * 32 + 32 + 32 * 16 + 16
    # the primary adds one gradient buffer; a further replica has no ring (2 versions) and no optimiser state
    assert 4 * n_par <= first - one <= 4 * n_par + 1024
    assert 3 * 4 * n_par <= first - more <= 3 * 4 * n_par + 4096
    for kw in (dict(replicas=9), dict(replicas=-1), dict(replicas=2, vertical_sync=True)):
        with pytest.raises(pd.PdError) as e:
            pd.pd_stage_query_bytes(pd.make_config(layers, minibatch=8, **kw))
        assert e.value.status == pd.PD_EINVAL
    with pytest.raises(pd.PdError):      # a further replica of a stage that is not replicated
        pd.pd_stage_replica_query_bytes(pd.make_config(layers, minibatch=8))
