"""sod2_run_static (the entry point that allocates nothing: split-K partials in the library's static device
buffer) against sod2_run with a workspace behind the arena, through the C ABI: bit-identical outputs on two
calls in a row, the second with a smaller input, with the automatic split-K choice and with forced
splits; a binding whose partial tiles exceed the static buffer, and graphs that need read-backs, are
refused with nothing launched."""
import numpy as np
import pytest

from workloads import configs

pytestmark = pytest.mark.gpu


def _bits(t):
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().copy()


def test_static_scratch_run_matches_workspace_run():
    import torch
    import paper_2403_00176_amd as S
    from paper_2403_00176_amd.session import Session
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    w = configs.config2(4, layers=2)
    ses = Session(w.graph)
    ses.upload_weights(w.make_weights())
    wptrs = [x.data_ptr() for x in ses.weights]
    stream = ses.stream.cuda_stream
    # (B*L, forced splits): the FFN2 contraction (k = 3072) of the first call splits k by itself;
    # the second call is smaller; then forced splits on every contraction
    for sym, splits in (({"B": 2, "L": 150}, 0), ({"B": 1, "L": 40}, 0), ({"B": 1, "L": 100}, 4), ({"B": 1, "L": 33}, 16)):
        print(f"case static scratch sym {sym} splits {splits}", flush=True)
        ins = ses.upload_inputs(w.make_inputs(0, sym))
        b = ses.bind(sym)
        if splits:
            S.sod2_binding_force_splits(b, splits)
        ref = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ins, ref)                                    # sod2_run, workspace behind the arena
        torch.cuda.synchronize()
        plan_bytes = S.sod2_binding_arena_bytes(b)[0]
        arena = torch.empty(max(plan_bytes, 256), dtype=torch.uint8, device=ses.device)   # no workspace
        b2 = ses.bind(sym)
        if splits:
            S.sod2_binding_force_splits(b2, splits)
        got = ses.alloc_outputs(ses.output_shapes(b2))
        for o in got:
            o.zero_()
        S.sod2_run_static(b2, arena.data_ptr(), arena.numel(), wptrs, [t.data_ptr() for t in ins],
                          [t.data_ptr() for t in got], stream)
        torch.cuda.synchronize()
        for r, g in zip(ref, got):
            assert np.array_equal(_bits(r), _bits(g)), (sym, splits)
        # without any workspace sod2_run does not split: its result differs from the split one in the last
        # bits somewhere, which shows the static buffer was in use above
        if splits:
            plain = ses.alloc_outputs(ses.output_shapes(b2))
            b3 = ses.bind(sym)
            S.sod2_binding_force_splits(b3, splits)
            S.sod2_run(b3, arena.data_ptr(), arena.numel(), wptrs, [t.data_ptr() for t in ins],
                       [t.data_ptr() for t in plain], stream)
            torch.cuda.synchronize()
            assert any(not np.array_equal(_bits(p), _bits(g)) for p, g in zip(plain, got))


def test_static_scratch_refusals():
    import torch
    import paper_2403_00176_amd as S
    from paper_2403_00176_amd.session import Session
    w = configs.config2(1, layers=1)
    ses = Session(w.graph)
    ses.upload_weights(w.make_weights())
    wptrs = [x.data_ptr() for x in ses.weights]
    sym = {"B": 4, "L": 400}                  # 1600 rows x 768 columns x 2 splits x 4 bytes = 9.8 MB > 8 MiB
    b = ses.bind(sym)
    S.sod2_binding_force_splits(b, 2)
    ins = ses.upload_inputs(w.make_inputs(0, sym))
    outs = ses.alloc_outputs(ses.output_shapes(b))
    for o in outs:
        o.fill_(7.0)
    arena = torch.empty(S.sod2_binding_arena_bytes(b)[0], dtype=torch.uint8, device=ses.device)
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_run_static(b, arena.data_ptr(), arena.numel(), wptrs, [t.data_ptr() for t in ins],
                          [t.data_ptr() for t in outs], ses.stream.cuda_stream)
    assert e.value.code == -10 and "static buffer holds 8388608" in str(e.value)
    torch.cuda.synchronize()
    assert all(bool((o == 7.0).all()) for o in outs)            # nothing was launched
    # a graph with Switch operators needs a read-back slot: refused
    g4 = configs.config4(1, layers=1)
    s4 = Session(g4.graph)
    s4.upload_weights(g4.make_weights())
    b4 = s4.bind({"L": 128})
    ins4 = s4.upload_inputs(g4.make_inputs(0, {"L": 128}))
    outs4 = s4.alloc_outputs(s4.output_shapes(b4))
    arena4 = torch.empty(S.sod2_binding_arena_bytes(b4)[0], dtype=torch.uint8, device=s4.device)
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_run_static(b4, arena4.data_ptr(), arena4.numel(), [x.data_ptr() for x in s4.weights],
                          [t.data_ptr() for t in ins4], [t.data_ptr() for t in outs4], s4.stream.cuda_stream)
    assert e.value.code == -6
