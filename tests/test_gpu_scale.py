"""Parity at the real layer shapes of the large workloads (1.3B, 7B, 14B-GQA), with one block and a short
sequence so that the fp64 CPU oracle finishes in seconds, and sampled rows of attention at the 128k
context length.  The full-size steps themselves are checked by invariants only."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import mt_inputs
import paper_2604_05091_amd as mt
from gpu_util import bf16_round, cosine, dev_bf16, host, ok, rel_l2
from test_gpu_step import check_against_oracle, gpu_step

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,T", [("1.3B", 128), ("7B", 96), ("14B", 72)])
def test_one_block_at_real_width_matches_oracle(orc64, name, T):
    shape, _, _ = mt_inputs.CONFIGS[name]
    shape = replace(shape, n_layers=1)
    params = mt_inputs.make_params(shape, seed=0)
    tok, lab = mt_inputs.make_batch(shape.vocab, 1, T, seed=1)
    print(f"[scale] {name}: hidden {shape.hidden} ffn {shape.ffn} heads {shape.n_q_heads}/{shape.n_kv_heads} T {T}", flush=True)
    loss, grads, _ = gpu_step(shape, 1, T, params, tok, lab)
    check_against_oracle(orc64, shape, 1, T, params, tok, lab, loss, grads)


def test_attention_rows_at_128k_context(orc64):
    """Forward output and dq of sampled query rows at T = 131072 (one sequence, 7B head layout reduced to
    2 query heads sharing nothing): each row needs only its own keys, so the oracle can do it row by row."""
    L = mt.lib()
    T, Hq, Hkv, hd = 131072, 2, 2, 128
    nq = Hq * hd
    ld = 3 * nq
    g = torch.Generator(device="cuda").manual_seed(5)
    qkv = (torch.randn((T, ld), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
    dout = torch.randn((T, nq), device="cuda", generator=g).to(torch.bfloat16)
    pq, pk, pv = qkv.data_ptr(), qkv.data_ptr() + 2 * nq, qkv.data_ptr() + 4 * nq
    O = torch.zeros((T, nq), dtype=torch.bfloat16, device="cuda")
    LSE = torch.zeros((1, Hq, T), dtype=torch.float32, device="cuda")
    scale = 1.0 / np.sqrt(hd)
    ok(L.mt_k_flash_fwd(O.data_ptr(), nq, LSE.data_ptr(), pq, ld, pk, ld, pv, ld, 1, T, Hq, Hkv, hd, scale, None))
    DELTA = torch.empty((1, Hq, T), dtype=torch.float32, device="cuda")
    DQKV = torch.zeros((T, ld), dtype=torch.bfloat16, device="cuda")
    ok(L.mt_k_flash_bwd(DQKV.data_ptr(), ld, DQKV.data_ptr() + 2 * nq, ld, DQKV.data_ptr() + 4 * nq, ld,
                        dout.data_ptr(), nq, pq, ld, pk, ld, pv, ld, O.data_ptr(), nq, LSE.data_ptr(),
                        DELTA.data_ptr(), 1, T, Hq, Hkv, hd, scale, None))
    for h in (0, 1):
        kh = qkv[:, nq + h * hd: nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
        vh = qkv[:, 2 * nq + h * hd: 2 * nq + (h + 1) * hd].float().cpu().numpy().astype(np.float64)
        for t in (0, 63, 64, 4095, 65535, 131071):
            qt = qkv[t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
            dat = dout[t, h * hd:(h + 1) * hd].float().cpu().numpy().astype(np.float64)
            a_ref, dq_ref = orc64.attention_row(qt, dat, kh[: t + 1], vh[: t + 1])
            a = O[t, h * hd:(h + 1) * hd].float().cpu().numpy()
            dq = DQKV[t, h * hd:(h + 1) * hd].float().cpu().numpy()
            assert rel_l2(a, a_ref) < 1e-2, (h, t, rel_l2(a, a_ref))
            if t == 0:      # a single visible key: softmax is constant, so dq vanishes (up to rounding of p - 1)
                assert np.max(np.abs(dq)) < 1e-5 and np.all(dq_ref == 0)
            else:
                assert rel_l2(dq, dq_ref) < 3e-2 and cosine(dq, dq_ref) > 0.999, (h, t, rel_l2(dq, dq_ref))
