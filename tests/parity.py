"""Runs the HIP path and the CPU oracle on the same host arrays and compares
them.  Used by the GPU parity tests."""
import numpy as np
import torch

import paper_2604_21335_amd as stc
from oracle import stc_oracle as O

TOL = 2e-3          # max abs error of the attention output vs the oracle (bf16 in, fp32 acc)
TIGHT = 1e-4        # what this build holds itself to on N(0,1)-like data


def to_dev_bf16(bits, dev="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)


def to_dev_u16(a, dev="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).to(dev)


def host_u16(t):
    return t.contiguous().cpu().numpy().view(np.uint16)


def host_bf16(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def run_hip(K, V, q, G, k_pages, logits=None, kcount=None, fixed_k=0, mask_in=None, cap=None,
            dev="cuda:0", global_k=None):
    """All inputs are host numpy arrays (bf16 as uint16 bits).  Returns host outputs."""
    B, Hkv, N, D = K.shape
    Hq = q.shape[1]
    c = stc.RoutedCache(B, Hq, Hkv, D, N, G, k_pages, v_cap_groups=cap, device=dev)
    c.vpacked.view(torch.int16).fill_(0x7FC0)            # poison: untouched slots stay NaN
    dK, dV, dq = to_dev_bf16(K, dev), to_dev_bf16(V, dev), to_dev_bf16(q, dev)
    c.build(dK, dV,
            logits=None if logits is None else torch.from_numpy(logits).to(dev),
            kcount=None if kcount is None or np.isscalar(kcount) else torch.from_numpy(
                np.ascontiguousarray(kcount, dtype=np.uint8)).to(dev),
            fixed_k=int(kcount) if np.isscalar(kcount) and kcount is not None else fixed_k,
            mask_in=None if mask_in is None else to_dev_u16(mask_in, dev), global_k=global_k)
    c.page_score.fill_(float("nan"))
    if k_pages < (N + 15) // 16:
        # the step as two calls (selection, attention) and as one: the same bits
        c.step(dq, one_call=False)
        torch.cuda.synchronize()
        two = (c.page_idx.clone(), c.out.clone(), c.page_score.clone())
        c.page_score.fill_(float("nan"))
        c.page_idx.fill_(-7)
        c.out.fill_(float("nan"))
        c.step(dq)
        torch.cuda.synchronize()
        assert torch.equal(two[0], c.page_idx), "page lists of the one-call step differ"
        assert torch.equal(two[1], c.out), "outputs of the one-call step differ"
        assert torch.equal(two[2].view(torch.int32), c.page_score.view(torch.int32))
    else:
        c.step(dq)
        torch.cuda.synchronize()
    return {
        "bounds": host_bf16(c.bounds_rows()), "bounds_raw": host_bf16(c.bounds), "mask": host_u16(c.mask),
        "tok_off": c.tok_off.cpu().numpy().view(np.uint32), "vpacked": host_bf16(c.vpacked),
        "dev_status": int(c.dev_status.item()), "page_idx": c.page_idx.cpu().numpy(),
        "page_score": c.page_score.cpu().numpy(), "out": c.out.cpu().numpy(), "cache": c,
    }


def run_oracle(K, V, q, G, k_pages, logits=None, kcount=None, mask_in=None, streams=None,
               global_k=None):
    """Oracle on every stream, or on the listed (b, h) streams only."""
    B, Hkv, N, D = K.shape
    Hq = q.shape[1]
    R = Hq // Hkv
    res = {}
    todo = streams if streams is not None else [(b, h) for b in range(B) for h in range(Hkv)]
    for (b, h) in todo:
        bounds = O.page_bounds(K[b, h])
        if mask_in is not None:
            m = np.asarray(mask_in[b, h], dtype=np.uint16) & np.uint16((1 << G) - 1)
        elif global_k is not None:
            m = O.route_mask_global(logits[b, h], N * int(global_k))
        else:
            kc = kcount if np.isscalar(kcount) else kcount[b, h]
            m = O.route_mask(logits[b, h], kc)
        off = O.token_offsets(m, G)
        packed = O.pack_values(V[b, h], m, off, G)
        qh = q[b, h * R:(h + 1) * R]
        NP = bounds.shape[0]
        if k_pages >= NP:
            score = None
            idx = np.arange(NP, dtype=np.int32)
        else:
            score = O.page_scores(qh, bounds)
            idx = O.select_pages(score, k_pages)
        out = O.decode_attention(qh, K[b, h], V[b, h], m, idx, G)
        res[(b, h)] = dict(bounds=bounds, mask=m, tok_off=off, vpacked=packed, page_score=score,
                           page_idx=idx, out=out)
    return res


def compare(hip, ora, Hq, Hkv, tol=TOL):
    """Bit-exact on everything integer / byte / index, tolerance on the output.
    Returns the max abs output error."""
    R = Hq // Hkv
    worst = 0.0
    for (b, h), o in ora.items():
        tag = "stream (%d,%d)" % (b, h)
        assert np.array_equal(hip["bounds"][b, h], o["bounds"]), tag + " bounds"
        assert np.array_equal(hip["mask"][b, h], o["mask"]), tag + " mask"
        assert np.array_equal(hip["tok_off"][b, h], o["tok_off"]), tag + " tok_off"
        tot = int(o["tok_off"][-1])
        if hip["dev_status"] == 0:
            assert np.array_equal(hip["vpacked"][b, h, :tot], o["vpacked"]), tag + " vpacked"
            # slots past the stream total are never written
            assert np.all(hip["vpacked"][b, h, tot:] == 0x7FC0), tag + " wrote past the total"
        if o["page_score"] is not None:
            assert np.array_equal(hip["page_score"][b, h].view(np.uint32),
                                  o["page_score"].view(np.uint32)), tag + " page_score bits"
        assert np.array_equal(hip["page_idx"][b, h], o["page_idx"]), tag + " page_idx"
        err = float(np.abs(hip["out"][b, h * R:(h + 1) * R].astype(np.float64) - o["out"]).max())
        assert err <= tol, "%s out: max abs err %.3e > %.1e" % (tag, err, tol)
        worst = max(worst, err)
    return worst
