"""The entry point that allocates no device memory (``qflash_attention_static``) against the
ordinary one (``qflash_attention``) and the oracle, through the C ABI: two calls in a row on one
stream, the second with a smaller input and other constants (the static table memory keeps the
first call's table), then the refusal of constants whose table exceeds the static memory.
"""
import ctypes

import numpy as np
import pytest

import oracle
from workloads import quantize_per_tensor

pytestmark = pytest.mark.gpu


def _case(shape, seed, gain):
    rng = np.random.default_rng(seed)
    Qf = rng.standard_normal(shape).astype(np.float32) * np.float32(gain)
    Kf = rng.standard_normal(shape).astype(np.float32)
    Vf = rng.standard_normal(shape).astype(np.float32)
    (Q, sQ), (K, sK), (V, _) = (quantize_per_tensor(x) for x in (Qf, Kf, Vf))
    return Q, K, V, oracle.derive_params(sQ, sK, shape[-1])


def test_static_entry_point_matches_ordinary_one_twice_in_a_row():
    import torch
    import paper_2604_25306_amd as qf
    assert torch.cuda.is_available(), "this test needs a GPU"
    lib = qf.load_library()
    dev = torch.device("cuda:0")
    with qf.Context(0) as ctx:
        handle = ctypes.c_void_p(ctx.handle)
        stream = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
        used_table = []
        # the second call is smaller (fewer heads, shorter sequence) and has coarser constants
        for shape, seed, gain, tile in (((3, 4, 197, 64), 11, 1.0, 64), ((2, 2, 70, 64), 12, 1.6, 64)):
            Q, K, V, p = _case(shape, seed, gain)
            x_p = -(-8 * p.s_inv >> p.x_shift)
            used_table.append(x_p + 16 <= 32 * 1024)
            lp = qf.QFlashParams(*p.astuple())
            tQ, tK, tV = (torch.from_numpy(x).to(dev) for x in (Q, K, V))
            outs = []
            for fn in (lib.qflash_attention_static, lib.qflash_attention):
                tO = torch.full(shape, 0x55, dtype=torch.int8, device=dev)
                print("call", fn.__name__, shape, "s_inv", p.s_inv, flush=True)
                rc = fn(handle, tQ.data_ptr(), tK.data_ptr(), tV.data_ptr(), tO.data_ptr(), None, 0, 0,
                        shape[0], shape[1], shape[2], shape[3], tile, ctypes.byref(lp), stream)
                assert rc == 0, qf.qflash_strerror(rc)
                outs.append(tO)
            torch.cuda.synchronize()
            a, b = (o.cpu().numpy() for o in outs)
            assert np.array_equal(a, b), "static entry point differs from qflash_attention: %s" % (shape,)
            ref = oracle.qflash_attention(Q, K, V, p, tile)
            assert np.array_equal(a, ref), "static entry point differs from the oracle: %s" % (shape,)
        assert all(used_table), "both cases are meant to run in table mode"


def test_static_entry_point_refuses_a_table_beyond_its_memory():
    import torch
    import paper_2604_25306_amd as qf
    assert torch.cuda.is_available(), "this test needs a GPU"
    dev = torch.device("cuda:0")
    shape = (1, 2, 100, 64)
    Q, K, V, _ = _case(shape, 13, 1.0)
    # a fine score scale: s_inv = 4500, table of 8 * 4500 bytes > 32 KiB
    p = oracle.derive_params(0.02, 1.0 / (0.02 * 4500 * 1.4426950408889634 / 8.0), 64)
    assert 8 * p.s_inv + 16 > 32 * 1024 and p.x_shift == 0
    lp = qf.QFlashParams(*p.astuple())
    tQ, tK, tV = (torch.from_numpy(x).to(dev) for x in (Q, K, V))
    tO = torch.full(shape, 0x55, dtype=torch.int8, device=dev)
    with qf.Context(0) as ctx:
        with pytest.raises(qf.QFlashError) as e:
            ctx.attention_static(tQ, tK, tV, tO, lp, 64)
        assert e.value.code == qf.ERR["SCRATCH"]
        torch.cuda.synchronize()
        assert bool((tO == 0x55).all()), "a refused call must not write"
        # without the table the same constants are accepted and need no static memory
        ctx.configure(qf.CFG_EXP_TABLE, 0)
        ctx.attention_static(tQ, tK, tV, tO, lp, 64)
        torch.cuda.synchronize()
        assert np.array_equal(tO.cpu().numpy(), oracle.qflash_attention(Q, K, V, p, 64))
