"""Helpers shared by the GPU parity tests: run a window of steps through the
HIP library (via the C ABI binding) and return numpy results; norm-wise
comparison against the oracle."""
from __future__ import annotations

import numpy as np


def to_dev(a, torch):
    """numpy -> cuda tensor; uint16 arrays are bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def run_window(X, W, batches, *, vocab_n, pad_id=0, k_steps=None, max_positions=None, u_total_cap=0,
               keep_H=True, keep_E=True, want_G=True, gram_obj=None, X_dev=None, W_dev=None,
               pass_E=True, foreign_buffers=False, profile=None, pseudo=False, wgrad_chunks=None,
               dense=False, resume=None, h_bf16=False, window_end=False):
    """batches: list of (ids int32 [m], dH float32 [m,d]).  Returns dict with per-step
    uniq/inverse/counts/E/H and the window's uniq_total/counts_total/G_total/dW.
    pass_E=False calls gram_encode_gather with E = NULL (no "E" in the result);
    foreign_buffers=True hands it copies of uniq / inverse instead of the buffers gram_unique
    wrote, which selects the two-kernel forward.  profile: kernel names whose launches are counted
    (result key "profile": name -> (launches, ms)).  pseudo=True also calls gram_pseudo_target
    and gram_gather after each accumulate (step keys "Ht", "loss", "H_tilde").  wgrad_chunks: list of
    (first_row, n_rows); before the full weight gradient each chunk is taken alone (key "dW_chunks")
    and all of them accumulated into one matrix (key "dW_chunked").  dense=True selects the
    one-row-per-ID buffer and exports through gram_flush64 (counts_total is then int64);
    resume=(ids, counts int64, G rows float32) is merged into the window with gram_window_import
    before the first step.  h_bf16=True asks for H in bf16 (returned widened to float32).
    window_end=True ends the window with the one call gram_window_end instead of
    gram_encoder_wgrad followed by gram_flush."""
    import torch
    from paper_2204_04179_amd import gram

    d_in, d = W.shape
    xw = gram.F32 if X.dtype == np.float32 else gram.BF16
    K = k_steps or len(batches)
    M_max = max_positions or max(1, max(b[0].size for b in batches))
    cfg = gram.make_config(vocab_n, d_in, d, M_max, K, pad_id, u_total_cap, xw, 1 if dense else 0, 0,
                           gram.BF16 if h_bf16 else gram.F32)
    h_dt = torch.bfloat16 if h_bf16 else torch.float32
    g = gram_obj or gram.Gram(cfg)
    if profile:
        g.profile_enable(profile, max_launches=256)
    Xd = X_dev if X_dev is not None else to_dev(X, torch)
    Wd = W_dev if W_dev is not None else to_dev(W, torch)
    cap_u = max(1, min(M_max, vocab_n))
    steps = []
    if resume is not None:
        r_ids, r_cnt, r_G = (torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in resume)
        g.window_import(r_ids, r_cnt, r_G, r_ids.numel())
    for k, (ids, dH) in enumerate(batches):
        m = int(ids.size)
        ids_d = torch.from_numpy(np.ascontiguousarray(ids.reshape(-1))).cuda()
        dH_d = torch.from_numpy(np.ascontiguousarray(dH.reshape(m, d))).cuda()
        uniq = torch.full((cap_u,), -7, dtype=torch.int32, device="cuda")
        counts = torch.full((cap_u,), -7, dtype=torch.int32, device="cuda")
        inverse = torch.full((max(1, m),), -7, dtype=torch.int32, device="cuda")
        u_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
        E = torch.full((cap_u, d), float("nan"), device="cuda")
        H = torch.full((max(1, m), d), float("nan"), dtype=h_dt, device="cuda")
        U = g.unique(ids_d, uniq, inverse, counts, u_dev, want_host_u=True)
        assert int(u_dev.item()) == U
        uq, inv = (uniq.clone(), inverse.clone()) if foreign_buffers else (uniq, inverse)
        g.encode_gather(Xd, Wd, uq, inv, u_dev, m, E if pass_E else None, H)
        g.grad_accumulate(dH_d, m, k)
        if pseudo:
            Ht = torch.full((cap_u, d), float("nan"), device="cuda")
            loss = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
            H2 = torch.full((max(1, m), d), float("nan"), dtype=h_dt, device="cuda")
            g.pseudo_target(E, Ht, loss)
            g.gather(Ht, inverse, m, H2)
        torch.cuda.synchronize()
        st = dict(U=U, uniq=uniq[:U].cpu().numpy(), counts=counts[:U].cpu().numpy(),
                  inverse=inverse[:m].cpu().numpy(),
                  uniq_tail_untouched=bool((uniq[U:] == -7).all().item()))
        if keep_E and pass_E:
            st["E"] = E[:U].cpu().numpy()
        if keep_H:
            st["H"] = H[:m].float().cpu().numpy()
        if pseudo:
            st["Ht"], st["loss"], st["H_tilde"] = Ht[:U].cpu().numpy(), float(loss.item()), H2[:m].float().cpu().numpy()
            st["Ht_tail_untouched"] = bool(torch.isnan(Ht[U:]).all().item())
        st["H_dev"], st["E_dev"], st["inverse_dev"] = H, E, inverse
        steps.append(st)
    chunk_out = {}
    if wgrad_chunks:
        acc = torch.full((d_in, d), float("nan"), device="cuda")
        singles = []
        for i, (a, nrows) in enumerate(wgrad_chunks):
            one = torch.full((d_in, d), float("nan"), device="cuda")
            g.encoder_wgrad_chunk(Xd, one, a, nrows, False)
            g.encoder_wgrad_chunk(Xd, acc, a, nrows, i > 0)
            singles.append(one)
        torch.cuda.synchronize()
        chunk_out = dict(dW_chunks=[t.cpu().numpy() for t in singles], dW_chunked=acc.cpu().numpy())
    dW = torch.full((d_in, d), float("nan"), device="cuda")
    if not window_end:
        g.encoder_wgrad(Xd, dW)
    cap_total = vocab_n if dense else (u_total_cap or max(1, min(K * M_max, vocab_n)))
    ut = torch.full((cap_total,), -7, dtype=torch.int32, device="cuda")
    ct = torch.full((cap_total,), -7, dtype=torch.int64 if dense else torch.int32, device="cuda")
    Gt = torch.full((cap_total, d), float("nan"), device="cuda") if want_G else None
    utd = torch.zeros(1, dtype=torch.int32, device="cuda")
    if window_end:
        assert not dense
        n = g.window_end(Xd, dW, ut, ct, Gt, utd, want_host_u=True)
    else:
        n = (g.flush64 if dense else g.flush)(ut, ct, Gt, utd, want_host_u=True)
    torch.cuda.synchronize()
    out = dict(steps=steps, dW=dW.cpu().numpy(), U_total=n, **chunk_out, uniq_total=ut[:n].cpu().numpy(),
               counts_total=ct[:n].cpu().numpy(), gram=g, X_dev=Xd, W_dev=Wd)
    assert int(utd.item()) == n
    if profile:
        out["profile"] = g.profile_read()
        g.profile_enable([])
    if want_G:
        out["G_total"] = Gt[:n].cpu().numpy()
        out["G_tail_untouched"] = bool(torch.isnan(Gt[n:]).all().item())
    return out


def rel_err(got, ref):
    """(max-norm, Frobenius) error of `got` relative to the size of `ref`."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0
    den_max = max(np.abs(ref).max(), 1e-300)
    den_f = max(np.sqrt((ref ** 2).sum()), 1e-300)
    return float(np.abs(got - ref).max() / den_max), float(np.sqrt(((got - ref) ** 2).sum()) / den_f)


def assert_close(got, ref, tol, what):
    """Norm-wise relative bound: max|got-ref| <= tol*max|ref| and ||got-ref||_F <= tol*||ref||_F."""
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    e_max, e_f = rel_err(got, ref)
    assert e_max <= tol and e_f <= tol, f"{what}: rel err max={e_max:.3e} fro={e_f:.3e} > {tol:g}"
    return e_max, e_f
