"""Parity at the benchmark's full size and launch configuration.

The LLaVA-1.5-13B workload (40 layers, 40 heads, d = 128, bf16, 35 + 576 + 128 prompt tokens) runs
at batch 32 through the same calls bench.py times (prefill per layer, then st3_decode_step with
deferred mass).  The oracle cannot afford 32 sequences, so it replays ONE sampled sequence in
full - every layer and head of its prefill and of the first decode steps - from the original
inputs, and everything the GPU produced for that sequence is compared with it.
"""
import numpy as np
import pytest
import torch

from gpu_util import DEV, assert_attention_close, assert_mass_close, assert_selection_matches, to_np64
from oracle import st3_oracle as orc
from paper_2412_20105_amd import pipeline
from workloads import get_workload

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


def _randn_bf16(gen, shape, sigma):
    return (torch.randn(shape, generator=gen, device=DEV, dtype=torch.float32) * sigma).to(torch.bfloat16)


@pytest.mark.parametrize("batch,sample_b", [(32, 17)])
def test_13b_full_shape_one_sequence_replayed_by_oracle(batch, sample_b):
    w = get_workload("llava15_13b")
    T = 3                                              # decode steps replayed (table keeps the full T = 512 schedule)
    keep_full = pipeline.keep_table_for(w)
    keep = [row[:T + 1] for row in keep_full]
    assert np.array_equal(np.array(keep_full), orc.schedule_for(w))
    gen = pipeline.Generation(w.layers, w.heads, w.head_dim, torch.bfloat16, batch, w.n_sys, w.n_vis, w.n_txt,
                              w.steps, keep_full, defer_mass=True, device=DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(20241227)
    shape_p = (batch, w.heads, w.n_prompt, w.head_dim)
    pre_host, gpu_out, gpu_mass, gpu_ids, gpu_rho = [], [], [], [], []
    for l in range(w.layers):
        if l % 8 == 0:
            print(f"full-size prefill layer {l}", flush=True)
        q, k, v = (_randn_bf16(g, shape_p, w.sigma) for _ in range(3))
        pre_host.append(tuple(x[sample_b:sample_b + 1].float().cpu().numpy() for x in (q, k, v)))
        out, mass = gen.prefill_layer(l, q, k, v)
        lc = gen.layers[l]
        gpu_out.append(to_np64(out[sample_b])); gpu_mass.append(to_np64(mass[sample_b]))
        gpu_ids.append(lc.ids[sample_b, :lc.h_vis].cpu().numpy())
        gpu_rho.append(to_np64(lc.score[sample_b, :lc.h_vis]))
    dec_dev = [_randn_bf16(g, (w.layers, 3, batch, w.heads, w.head_dim), w.sigma) for _ in range(T)]
    dec_host = [d[:, :, sample_b:sample_b + 1].float().cpu().numpy() for d in dec_dev]
    step_out, step_ids, step_mass_prev = [], [], []
    for t in range(1, T + 1):
        outs = gen.decode_step(t, dec_dev[t - 1])
        torch.cuda.synchronize()
        step_out.append(to_np64(outs[:, sample_b]))
        step_ids.append([gen.layers[l].ids[sample_b, :gen.layers[l].h_vis].cpu().numpy() for l in range(w.layers)])
        # with deferred mass, lc.mass now holds the PREVIOUS step's mass (in that step's order)
        step_mass_prev.append([to_np64(gen.layers[l].mass[sample_b]) for l in range(w.layers)])
    final_mass = [to_np64(gen.finalize_mass(l)[sample_b]) for l in range(w.layers)]
    torch.cuda.synchronize()
    for l in range(w.layers):
        assert gen.layers[l].kv_len.cpu().tolist() == [orc.kv_len(w.n_sys, keep[l][T], w.n_txt, T)] * batch

    # ---- the oracle replays the sampled sequence from the original inputs -----------------------
    print("oracle replay of one sequence (prefill of 40 layers, then decode steps)", flush=True)
    ref = orc.Generation(w.layers, w.heads, w.head_dim, w.n_sys, w.n_vis, w.n_txt, np.array(keep))
    r = ref.prefill(lambda l: pre_host[l])
    alive = True
    for l in range(w.layers):
        if l > 0 and keep[l][0] < keep[l - 1][0]:
            same = assert_selection_matches(gpu_ids[l], r["mass"][l - 1][0], r["ids"][l - 1][0], keep[l][0],
                                            f"prefill select l={l}")
            if not same:
                alive = False                        # a near-tie went the other way: later values differ legitimately
        if not alive:
            break
        assert np.array_equal(gpu_ids[l], r["ids"][l][0])
        assert_attention_close(gpu_out[l], r["out"][l][0], "bf16", f"prefill out l={l}")
        assert_mass_close(gpu_mass[l], r["mass"][l][0], f"prefill mass l={l}")
        assert_mass_close(gpu_rho[l], ref.rho[l][0], f"ranking column l={l}")
    assert alive, "prefill selection diverged on a near-tie; pick another sampled sequence"
    ok = np.ones(w.layers, bool)
    prev = None
    for t in range(1, T + 1):
        rho_before = [ref.rho[l][0].copy() for l in range(w.layers)]
        ids_before = [ref.ids[l][0].copy() for l in range(w.layers)]
        s = ref.decode_step(lambda l: (dec_host[t - 1][l, 0], dec_host[t - 1][l, 1], dec_host[t - 1][l, 2]))
        cur = []
        for l in range(w.layers):
            ids = step_ids[t - 1][l]
            if ok[l]:
                ok[l] = assert_selection_matches(ids, rho_before[l], ids_before[l], keep[l][t], f"t={t} l={l}")
            if not ok[l]:
                cur.append(None)
                continue
            assert_attention_close(step_out[t - 1][l], s["out"][l][0], "bf16", f"decode out t={t} l={l}")
            pos = np.searchsorted(s["ids"][l][0], ids)
            cur.append(s["mass"][l][0][pos])
            if prev is not None and prev[l] is not None:
                assert_mass_close(step_mass_prev[t - 1][l][:len(prev[l])], prev[l], f"deferred mass t={t - 1} l={l}")
        prev = cur
    for l in range(w.layers):
        if prev[l] is not None:
            assert_mass_close(final_mass[l][:len(prev[l])], prev[l], f"final mass l={l}")
    assert ok.mean() > 0.8
