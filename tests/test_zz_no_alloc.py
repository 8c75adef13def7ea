"""pc_prefill_attn_static: the attention call for callers that cannot allocate (its split-KV partials live in a
fixed array inside the library's device code).  Its output must be that of pc_prefill_attn, bit for bit, and within
the oracle's tolerance; two calls in a row, the second smaller, share the array."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from gpu_util import attn_errors, to_f64
import oracle
from paper_2311_04934_amd import binding as pcb

pytestmark = pytest.mark.gpu


def _inputs(seed, n_q, n_kv, hq, hkv, d, dev):
    g = torch.Generator().manual_seed(seed)
    K = torch.randn((n_kv, hkv, d), generator=g).to(torch.bfloat16)
    V = torch.randn((n_kv, hkv, d), generator=g).to(torch.bfloat16)
    Q = torch.randn((n_q, hq, d), generator=g).to(torch.bfloat16)
    # keys at positions 0..n_kv-1 in shuffled buffer order; the queries sit at the last n_q positions
    perm = torch.randperm(n_kv, generator=g)
    pos = perm.to(torch.int32)
    q_pos = torch.arange(n_kv - n_q, n_kv, dtype=torch.int32)
    return Q, K, V, pos, q_pos


def test_static_scratch_call_matches_the_allocating_call_twice_in_a_row():
    dev = torch.device("cuda:0")
    hq, hkv, d = 8, 2, 128
    pc = pcb.PromptCache(1, hq, hkv, d, pcb.PC_BF16, max_pos=8192, pool_bytes=1 << 20)
    try:
        for seed, n_q, n_kv in ((11, 100, 3000), (12, 40, 1000)):    # the second call is the smaller one
            Q, K, V, pos, q_pos = _inputs(seed, n_q, n_kv, hq, hkv, d, dev)
            dQ, dK, dV, dpos, dqpos = (t.to(dev) for t in (Q, K, V, pos, q_pos))
            ref = torch.full((n_q, hq, d), float("nan"), dtype=torch.bfloat16, device=dev)
            got = torch.full_like(ref, float("nan"))
            pc.pc_prefill_attn(0, dQ, dqpos, dK, dV, dpos, n_kv, ref)
            splits_ref = pc.pc_last_attn_launch()[0]
            pc.pc_prefill_attn_static(0, dQ, dqpos, dK, dV, dpos, n_kv, got)
            splits_got = pc.pc_last_attn_launch()[0]
            torch.cuda.synchronize()
            assert splits_ref == splits_got and splits_got > 1, (splits_ref, splits_got)   # the scratch is really used
            assert torch.equal(ref.cpu().view(torch.int16), got.cpu().view(torch.int16)), (seed, n_q, n_kv)
            want = oracle.attn(to_f64(Q), q_pos.numpy(), to_f64(K), to_f64(V), pos.numpy(), 10000.0)
            err, rel = attn_errors(got.cpu(), want)
            assert err <= 2e-2 and rel <= 1e-2, (seed, err, rel)
    finally:
        pc.close()


def test_static_scratch_call_refuses_partials_beyond_its_array_and_enqueues_nothing():
    dev = torch.device("cuda:0")
    hq, hkv, d = 8, 1, 128
    n_q, n_kv = 249 * 32, 512      # 249 row blocks -> 2 KV splits -> 2 * 7968 * 8 * 264 bytes > 32 MiB
    pc = pcb.PromptCache(1, hq, hkv, d, pcb.PC_BF16, max_pos=16384, pool_bytes=1 << 20)
    try:
        Q = torch.zeros((n_q, hq, d), dtype=torch.bfloat16, device=dev)
        K = torch.zeros((n_kv, hkv, d), dtype=torch.bfloat16, device=dev)
        pos = torch.arange(n_kv, dtype=torch.int32, device=dev)
        q_pos = torch.full((n_q,), n_kv, dtype=torch.int32, device=dev)
        out = torch.full((n_q, hq, d), 3.0, dtype=torch.bfloat16, device=dev)
        with pytest.raises(pcb.PcError) as e:
            pc.pc_prefill_attn_static(0, Q, q_pos, K, K, pos, n_kv, out)
        assert e.value.status == -5      # PC_E_CAPACITY
        torch.cuda.synchronize()
        assert bool((out == 3.0).all())
        pc.pc_prefill_attn(0, Q, q_pos, K, K, pos, n_kv, out)    # the allocating call takes the same shape
        torch.cuda.synchronize()
        assert pc.pc_last_attn_launch()[0] == 2 and bool((out == 0.0).all())
    finally:
        pc.close()
