"""plt_use_graph: the decode step replayed as one HIP graph gives the eager step's bits, on every replay, with the
program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2510_24824_amd import binding as B, synth
from tests.helpers import lively_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,L,moe,n_seq,n_prompt",
                         [(B.PLT_BF16, 3, False, 3, 70), (B.PLT_F32, 2, False, 3, 70), (B.PLT_BF16, 2, True, 3, 70),
                          # one sequence, 600 tokens: the attention splits every stream over two workgroups, whose records
                          # the last one to finish merges (a device counter that must be back at zero for every replay)
                          (B.PLT_BF16, 2, False, 1, 600)],
                         ids=["bf16-L3", "f32-L2", "bf16-moe", "bf16-L2-split-streams"])
def test_graph_replay_equals_eager_steps(dtype, L, moe, n_seq, n_prompt):
    if moe:
        shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64, ffn_hidden=64,
                                 vocab=300, n_loops=L, window=5, n_experts=8, top_k=2)
    else:
        shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64, ffn_hidden=192,
                                 vocab=300, n_loops=L, window=5)
    weights = lively_weights(shape, 3, bf16=dtype == B.PLT_BF16, std=0.05, router_std=0.5 if moe else None)
    cfg = B.make_config(shape, dtype=dtype)
    prompts = torch.from_numpy(np.ascontiguousarray(synth.token_ids((n_seq, n_prompt), shape.vocab, 4), np.int32))
    side = torch.cuda.Stream()                       # stream capture needs a stream of its own (not the NULL stream)
    with torch.cuda.stream(side):
        blob = B.pack_weights(cfg, weights)
        model = B.Model(cfg, blob)
        steps = 9

        def run(graph):
            model.use_graph(graph)
            kv = B.KV(model, n_seq, n_prompt + 30)
            nxt, _ = kv.prefill(prompts.cuda())
            out = []
            tok = nxt.clone()
            for i in range(steps):
                n1, lg = kv.decode_step(tok)
                # the program's own eager work between replays: device arithmetic, a copy to the host, a synchronisation
                junk = (lg * 2).sum().item()
                out.append((n1.cpu().numpy().copy(), lg.cpu().numpy().copy(), kv.get_hidden().copy(), junk))
                torch.cuda.synchronize()
                tok.copy_(n1)                         # same token buffer every step: the graph is captured once
            assert kv.position == n_prompt + steps
            kv.close()
            return out

        eager = run(False)
        replay = run(True)
        model.use_graph(False)
        for i, (e, r) in enumerate(zip(eager, replay)):
            assert np.array_equal(e[0], r[0]), i
            assert np.array_equal(e[1], r[1]), i      # every replay: the eager step's logits bit for bit
            assert np.array_equal(e[2], r[2]), i
        model.close()
    torch.cuda.synchronize()


def test_graph_on_the_null_stream_is_refused_without_side_effects():
    shape = synth.TINY
    weights = synth.make_weights(shape, 1, bf16=False)
    cfg = B.make_config(shape, dtype=B.PLT_F32)
    model = B.Model(cfg, B.pack_weights(cfg, weights))        # torch's default stream = the NULL stream
    kv = B.KV(model, 1, 20)
    tok, _ = kv.prefill(torch.from_numpy(np.ascontiguousarray(synth.token_ids((1, 8), shape.vocab, 2), np.int32)).cuda())
    tok = tok.clone()
    carry = kv.get_carry()
    _, lg0 = kv.decode_step(tok)
    lg0 = lg0.cpu().numpy().copy()
    kv.set_position(8); kv.set_carry(carry)                    # back to the state before that step
    model.use_graph(True)
    with pytest.raises(B.PltError) as e:
        kv.decode_step(tok)
    assert e.value.code == -4 and kv.position == 8
    model.use_graph(False)
    _, lg1 = kv.decode_step(tok)                               # nothing was launched, nothing moved: the same step again
    assert np.array_equal(lg0, lg1.cpu().numpy())
    kv.close(); model.close()
