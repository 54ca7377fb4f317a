"""The library neither allocates nor synchronises, so a training step and a decode step can be
captured into a HIP graph.  Every replay is checked against the eager result, with eager work and
synchronisations between the replays."""
import pytest
import torch

from paper_2506_06266_amd import binding as cb
from paper_2506_06266_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_training_and_decode_steps_replay_from_a_graph():
    print("case graph capture: ragged attention fwd+bwd, kl_ragged loss, decode_small", flush=True)
    a = synth.attn_inputs(synth.ATTN_CONFIGS["ragged"], DEV)
    kcfg = synth.KL_CONFIGS["kl_ragged"]
    kl = synth.kl_inputs(kcfg, DEV)
    dcfg = synth.DECODE_CONFIGS["decode_small"]
    dc = synth.decode_inputs(dcfg, DEV)
    pk = synth.attn_packed_inputs(synth.PACKED_CONFIGS["ragged_packed"], DEV)
    pmax = synth.PACKED_CONFIGS["ragged_packed"].max_len

    def step(out):
        o, lse = cb.cart_attn_fwd(a["q"], a["k_own"], a["v_own"], a["z_k"], a["z_v"], o=out.get("o"), lse=out.get("lse"))
        g = cb.cart_attn_bwd(a["q"], a["k_own"], a["v_own"], a["z_k"], a["z_v"], o, lse, a["d_o"], n_frozen=1,
                             d_q=out.get("dq"), d_k_own=out.get("dk"), d_v_own=out.get("dv"),
                             d_z_k=out.get("dzk"), d_z_v=out.get("dzv"))
        loss, dl = cb.cart_distill_kl_fwd_bwd(kl["logits"], kl["teacher_idx"], kl["teacher_logp"], kcfg.scale,
                                              d_logits=out.get("dl"), loss=out.get("loss"))
        do, dlse = cb.cart_decode(dc["q"], dc["z_k"], dc["z_v"], dc["k_own"], dc["v_own"], dc["cu_lens"],
                                  dcfg.max_len, o=out.get("do"), lse=out.get("dlse"))
        po, plse = cb.cart_attn_varlen_fwd(pk["q"], pk["k_own"], pk["v_own"], pk["z_k"], pk["z_v"], pk["cu_seqlens"],
                                           pmax, o=out.get("po"), lse=out.get("plse"))
        pg = cb.cart_attn_varlen_bwd(pk["q"], pk["k_own"], pk["v_own"], pk["z_k"], pk["z_v"], pk["cu_seqlens"], pmax,
                                     po, plse, pk["d_o"], d_q=out.get("pdq"), d_k_own=out.get("pdk"),
                                     d_v_own=out.get("pdv"), d_z_k=out.get("pdzk"), d_z_v=out.get("pdzv"))
        return dict(o=o, lse=lse, dq=g[0], dk=g[1], dv=g[2], dzk=g[3], dzv=g[4], loss=loss, dl=dl, do=do, dlse=dlse,
                    po=po, plse=plse, pdq=pg[0], pdk=pg[1], pdv=pg[2], pdzk=pg[3], pdzv=pg[4])

    eager = {k: v.clone() for k, v in step({}).items()}
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        bufs = step({})                      # warm-up on the capture stream; also the output buffers
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(bufs)
    torch.cuda.synchronize()
    for replay in range(3):
        for v in bufs.values():
            v.zero_()                        # eager work between replays: every output is rebuilt
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(bufs[k], eager[k]), (replay, k)
        cb.cart_attn_fwd(a["q"], a["k_own"], a["v_own"], a["z_k"], a["z_v"])     # eager call in between
        torch.cuda.synchronize()
