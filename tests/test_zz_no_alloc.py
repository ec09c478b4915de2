"""The decode step on the library's built-in scratch memory (no workspace argument, no device allocation)
against the ordinary entry point, through the C ABI: two calls in a row, the second on a smaller batch."""
import numpy as np
import pytest

from paper_2506_24119_amd import inputs as si

pytestmark = pytest.mark.gpu


def test_static_workspace_step_equals_the_ordinary_step():
    import torch
    from paper_2506_24119_amd import binding as sb
    sb.load_library()
    g = si.ModelGeometry("g4-qknorm", 2, 256, 8, 2, 128, 640, 2048, 1e6, qk_norm=True)
    w = si.make_weights(g, seed=51)
    B = 6
    prompts = si.make_prompts(g.vocab, B, 3, 70, seed=52)
    forced = si.make_forced_tokens(g.vocab, B, 2, seed=53)
    ids = np.arange(B, dtype=np.int32)

    def session():
        return sb.Session(g, sb.weights_to_device(w), 64, B, 8, 512, 128, page_order=si.make_page_order(64, 7))

    ref, sta = session(), session()
    assert sb.spiral_workspace_bytes(sta.model, B, 128) <= sb.spiral_static_workspace_bytes()
    ref.prefill(ids, prompts)
    sta.prefill(ids, prompts)
    # first call: the whole batch; second call: a smaller one (three of the sequences, another order)
    for k, sub in enumerate((ids, np.array([4, 0, 2], dtype=np.int32))):
        tin = torch.from_numpy(np.ascontiguousarray(forced[k][sub])).cuda()
        want = ref.new_logits(len(sub))
        got = torch.full_like(want, float("nan"))
        ref.decode_step(sub, tin, want)
        sb.spiral_decode_step_static(sta.model, sta.pool, sub, tin, got)
        torch.cuda.synchronize()
        assert torch.isfinite(want).all()
        assert torch.equal(got, want), f"call {k}: max diff {(got - want).abs().max().item()}"
        assert [sb.spiral_seq_len(sta.pool, int(i)) for i in ids] == [sb.spiral_seq_len(ref.pool, int(i)) for i in ids]
    ref.close(); sta.close()


def test_static_workspace_step_rejects_what_does_not_fit():
    import torch
    from paper_2506_24119_amd import binding as sb
    g = si.ModelGeometry("wide", 1, 1024, 8, 8, 128, 1024, 2048, 1e6, qk_norm=True)      # 64 rows x 16 K splits of qkv alone: 12 MiB
    w = si.make_weights(g, seed=54)
    B = 64
    s = sb.Session(g, sb.weights_to_device(w), B + 2, B, 1, 256, 16)
    ids = np.arange(B, dtype=np.int32)
    s.prefill(ids, si.make_prompts(g.vocab, B, 2, 2, seed=55))
    assert sb.spiral_workspace_bytes(s.model, B, 16) > sb.spiral_static_workspace_bytes()
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    with pytest.raises(sb.SpiralError) as e:
        sb.spiral_decode_step_static(s.model, s.pool, ids, tok, s.new_logits(B))
    assert e.value.code == sb.SPIRAL_ERR_OOM_KV and "built-in scratch" in str(e.value)
    assert sb.spiral_seq_len(s.pool, 0) == 2 and sb.spiral_kv_free_pages(s.pool) == 2
    s.close()
