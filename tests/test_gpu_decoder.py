"""Config 5 on the GPU against the oracle: prompt pass, decode steps over the KV cache in the arena,
arg-max, with teacher forcing (the GPU run is fed the oracle's token at every step, so one flipped
near-tie cannot derail the comparison).  Tolerance: max |gpu - oracle| / max |oracle| <= 2e-2 per
logits row (bf16 storage, fp32 accumulation).  The arg-max is compared where the oracle's margin
between its two best logits is clear of that tolerance; elsewhere the GPU's choice must be one of
the near-best candidates."""
import numpy as np
import pytest

from oracle import rdp as R, plan as P, arena as A, execute, ops as O
from workloads import configs

pytestmark = pytest.mark.gpu
TOL = 2e-2


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def _oracle_sequence(w, W, plans, prompt, steps, exact=False, feed=None):
    """The oracle's prompt pass and decode steps.  ``feed``: the token given to decode step t (teacher
    forcing with another run's tokens); by default the run's own greedy token.  ``exact``: the float64
    definition without rounding of operator results to the storage type."""
    gp, gd = w.prefill, w.decode
    # weights rounded to their storage type once, not once per step
    Wr = {n: O.round_to(np.asarray(v, np.float64), w.dtype) for n, v in W.items()}
    r = execute.run(gp, plans["prefill"].order, w.weights_for(gp, Wr),
                    {gp.tensor_id("ids"): prompt, gp.tensor_id("pos"): np.arange(len(prompt))}, exact=exact,
                    round_weights=False)
    logits = [r.values[gp.tensor_id("logits")][0]]
    toks = [int(r.values[gp.tensor_id("next")][0])]
    state = r.state
    Wd = w.weights_for(gd, Wr)
    for t in range(steps):
        tok = toks[-1] if feed is None else feed[t]
        rd = execute.run(gd, plans["decode"].order, Wd,
                         {gd.tensor_id("ids"): np.array([tok]), gd.tensor_id("pos"): np.array([len(prompt) + t])},
                         state=state, exact=exact, round_weights=False)
        state = rd.state
        logits.append(rd.values[gd.tensor_id("logits")][0])
        toks.append(int(rd.values[gd.tensor_id("next")][0]))
    return logits, toks, state


def _check_token(row_ref, tok_gpu, tok_ref):
    scale = np.abs(row_ref).max()
    top = np.sort(row_ref)[-2:]
    if top[1] - top[0] > 2 * TOL * scale:
        assert tok_gpu == tok_ref
    else:
        assert row_ref[tok_gpu] >= top[1] - 2 * TOL * scale


def _run_decoder(S, w, W, seq, steps, check_structure=True, exact_taps=True):
    import torch
    from paper_2403_00176_amd.session import DecoderSession, to_host
    plans = {n: P.build_plan(g, R.RDP(g).analyse()) for n, g in (("prefill", w.prefill), ("decode", w.decode))}
    ses = DecoderSession(w.prefill, w.decode, w.t_max)
    ses.upload_weights(W)
    torch.cuda.synchronize()
    for prompt in seq:
        Pn = len(prompt)
        print(f"case {w.name} P={Pn} steps={steps}", flush=True)
        ref_logits, ref_toks, ref_state = _oracle_sequence(w, W, plans, prompt, steps)
        # the same sequence by the plain float64 definition (no rounding of operator results), fed the same tokens
        exact_state = _oracle_sequence(w, W, plans, prompt, steps, exact=True, feed=ref_toks)[2] if exact_taps else ref_state
        ses.start(Pn, w.vocab)
        if check_structure:
            assert S.sod2_binding_dump(ses.b_pre) == A.dump(A.bind(plans["prefill"], {"P": Pn}))
        ses.prefill(torch.from_numpy(np.asarray(prompt, dtype=np.int64)).to(ses.device))
        for t in range(steps):
            with torch.cuda.stream(ses.stream):
                ses.tokens[Pn + t] = ref_toks[t]             # teacher forcing
            b = ses.decode(t)
            if check_structure:
                assert S.sod2_binding_dump(b) == A.dump(A.bind(plans["decode"], {"P": Pn, "t": t}))
        torch.cuda.synchronize()
        got = to_host(ses.logits[:steps + 1])
        toks = ses.tokens.cpu().numpy()
        for t in range(steps + 1):
            e = rel_err(got[t], ref_logits[t])
            assert np.isfinite(got[t]).all() and e <= TOL, (Pn, t, e)
            if t < steps:                                    # token P+t was overwritten by the forced one
                continue
            _check_token(ref_logits[t], int(toks[Pn + t]), ref_toks[t])
        # the cache in the arena's session region against the oracle's state
        bd = A.bind(plans["decode"], {"P": Pn, "t": max(steps - 1, 0)})
        rows = Pn + steps
        errs, errs_exact, noise = {}, {}, {}
        for tid, (off, nbytes) in bd.session.items():
            name = w.decode.tensors[tid].name
            hidden = ref_state[name].shape[1]
            raw = ses.arena[off:off + rows * hidden * 2].view(torch.bfloat16).view(rows, hidden)
            got_rows = to_host(raw)
            errs[name] = rel_err(got_rows, ref_state[name][:rows])
            errs_exact[name] = rel_err(got_rows, exact_state[name][:rows])
            noise[name] = rel_err(ref_state[name][:rows], exact_state[name][:rows])
        print("cache max rel err per layer, library vs float64 definition / library vs rounded oracle / rounded oracle vs float64:",
              " ".join(f"{k}={errs_exact[k]:.1e}/{errs[k]:.1e}/{noise[k]:.1e}" for k in errs), flush=True)
        for name in errs:
            # Cache rows are taps on the way, not graph outputs.  Deep layers carry the storage roundings of
            # every block before them: the unfused oracle (one rounding per operator) is itself up to 1.8e-2
            # away from the float64 definition at layer 23, so the distance between two correctly rounded
            # executions can reach the sum of both.  The bar of the outputs is held against the definition,
            # for every layer; the distance to the rounded oracle is printed above.
            assert errs_exact[name] <= TOL, (name, errs_exact[name])
    return ses, plans


def test_decoder_small_widths(S_lib):
    """Small widths, ragged prompt lengths (P not a multiple of 8: scalar-load attention paths)."""
    w = configs.decoder(layers=2, hidden=128, heads=4, ffn=256, vocab=500, p_range=(4, 40), t_max=8)
    W = w.make_weights_by_name()
    seq = [w.make_prompt(0)[:5] % 500, w.make_prompt(1)[:33] % 500, w.make_prompt(2)[:40] % 500]
    _run_decoder(S_lib, w, W, seq, steps=8)


def test_decoder_full_widths_two_layers(S_lib):
    """Config 5's widths (hidden 1024, 16 heads, FFN 4096, vocab 32000) on 2 layers."""
    w = configs.decoder(layers=2, n_prompts=2)
    W = w.make_weights_by_name()
    seq = [w.make_prompt(0)[:64], w.make_prompt(1)[:121]]
    ses, plans = _run_decoder(S_lib, w, W, seq, steps=6)
    # incremental == full recompute on the GPU itself: decode logits at step t against the prompt
    # graph run on the whole prefix
    import torch
    from paper_2403_00176_amd.session import to_host
    Pn, steps = len(seq[1]), 6
    toks = ses.tokens[:Pn + steps].clone()
    inc = to_host(ses.logits[steps])
    torch.cuda.synchronize()
    ses.start(Pn + steps, w.vocab)
    ses.prefill(toks)
    torch.cuda.synchronize()
    assert rel_err(to_host(ses.logits[0]), inc) <= TOL


def test_config5_full_depth(S_lib):
    """All 24 layers: the shortest prompt of the benchmark's draw list and three decode steps."""
    w = configs.config5()
    W = w.make_weights_by_name()
    i = int(np.argmin(w.prompts))
    _run_decoder(S_lib, w, W, [w.make_prompt(i)], steps=3)


def test_longest_prompt_and_last_decode_steps(S_lib):
    """Config 5's widths on 2 layers with the longest prompt the config allows (P = 512: several query tiles in
    the prompt pass) and all 256 teacher-forced decode steps, so that the last steps run against cache lengths
    762 .. 767; every step's logits are compared, and the cache rows at the end."""
    w = configs.decoder(layers=2, n_prompts=4)
    W = w.make_weights_by_name()
    prompt = np.concatenate([w.make_prompt(i) for i in range(4)])
    assert len(prompt) >= 512
    _run_decoder(S_lib, w, W, [prompt[:512]], steps=256, check_structure=False, exact_taps=False)


def test_config5_full_depth_mid_prompt(S_lib):
    """All 24 layers with a prompt of mid length (P ~ 300) and two decode steps."""
    w = configs.config5()
    W = w.make_weights_by_name()
    i = int(np.argsort(w.prompts)[len(w.prompts) // 2])
    _run_decoder(S_lib, w, W, [w.make_prompt(i)], steps=2)


def test_free_running_generation_is_deterministic(S_lib):
    """Greedy generation without teacher forcing: the token written by step t is read by step t+1
    on the device (no host round trip); two runs give identical tokens."""
    import torch
    from paper_2403_00176_amd.session import DecoderSession
    w = configs.decoder(layers=2, hidden=256, heads=4, ffn=512, vocab=1000, p_range=(8, 64), t_max=16)
    ses = DecoderSession(w.prefill, w.decode, w.t_max)
    ses.upload_weights(w.make_weights_by_name())
    prompt = torch.from_numpy(np.asarray(w.make_prompt(0)[:20] % 1000, dtype=np.int64)).to(ses.device)
    torch.cuda.synchronize()
    runs = []
    for _ in range(2):
        ses.start(20, w.vocab)
        ses.prefill(prompt)
        for t in range(w.t_max):
            ses.decode(t)
        torch.cuda.synchronize()
        runs.append(ses.tokens.cpu().numpy().copy())
    assert np.array_equal(runs[0], runs[1])
    assert (runs[0][20:] >= 0).all() and (runs[0][20:] < 1000).all()


def test_decode_replay_matches_eager_steps(S_lib):
    """The decode steps as replays of one captured HIP graph (step counter on the device) against the
    same steps bound and launched one by one: same tokens, same logits bit for bit.  The graph is
    replayed in several batches with eager work (a prompt pass of another length, synchronisations)
    between them, and every batch is checked."""
    import torch
    from paper_2403_00176_amd.session import DecoderSession
    w = configs.decoder(layers=2, n_prompts=2, t_max=24)
    ses = DecoderSession(w.prefill, w.decode, w.t_max)
    ses.upload_weights(w.make_weights_by_name())
    Pn = 77
    prompt = torch.from_numpy(np.asarray(w.make_prompt(0)[:Pn], dtype=np.int64)).to(ses.device)
    torch.cuda.synchronize()
    ses.start(Pn, w.vocab)
    ses.prefill(prompt)
    for t in range(w.t_max):
        ses.decode(t)
    torch.cuda.synchronize()
    eager_tokens = ses.tokens.cpu().numpy().copy()
    eager_logits = ses.logits.view(torch.int16).cpu().numpy().copy()
    other = DecoderSession(w.prefill, w.decode, w.t_max)
    other.pre.weights = other.dec.weights = ses.pre.weights
    ses.start(Pn, w.vocab)
    ses.prefill(prompt)
    done = 0
    for n in (1, 5, 2, 16):
        ses.decode_replay(done, n)
        done += n
        torch.cuda.synchronize()
        assert np.array_equal(ses.tokens.cpu().numpy()[:Pn + done + 1], eager_tokens[:Pn + done + 1]), done
        assert np.array_equal(ses.logits.view(torch.int16).cpu().numpy()[:done + 1], eager_logits[:done + 1]), done
        other.start(64 + done // 2, w.vocab)                  # eager work between the replays
        other.prefill(prompt[:64 + done // 2])
        torch.cuda.synchronize()
    assert done == w.t_max
    with pytest.raises(S_lib.Sod2Error):
        ses.decode_replay(w.t_max - 1, 2)
