"""Lock-step parity driver: the HIP path and the CPU oracle advance one speculative step at a time on the same
committed tokens.  Floating-point outputs are compared element by element; integer decisions must be equal
wherever the oracle's own decision margin exceeds `margin_thr` (a differing near-tie is counted as excused and
the oracle adopts the GPU's choice so that both keep the same state)."""
from dataclasses import dataclass, field
from typing import List

import numpy as np

import paper_2401_15077_amd as pkg


@dataclass
class Stats:
    steps: int = 0
    emitted: int = 0
    max_logit_err: float = 0.0
    max_feat_err: float = 0.0
    max_draft_logit_err: float = 0.0
    max_draft_feat_err: float = 0.0
    excused_tree_slots: int = 0
    excused_accepts: int = 0
    lens: List[int] = field(default_factory=list)

    @property
    def tau(self):
        return self.emitted / max(1, self.steps)


def check_prefill(eng, orc, prompt, tol, margin_thr=2e-2, seq=0):
    first_g = eng.prefill(seq, prompt)
    first_o = orc.prefill(prompt)
    lg = eng.get_buffer(pkg.BUF_VANILLA_LOGITS, seq)
    err = float(np.abs(lg - orc.prefill_logits[-1]).max())
    assert err <= tol, f"prefill logits differ by {err}"
    # the features of every row of the prompt's last pass (the whole prompt when it fits one pass)
    pf = eng.get_buffer(pkg.BUF_PREFILL_FEATURES, seq)
    ferr = float(np.abs(pf - orc.prefill_features[len(prompt) - pf.shape[0]:]).max())
    assert ferr <= tol, f"prefill features differ by {ferr}"
    if first_g != first_o:
        if orc.T == 0.0:
            lo = orc.prefill_logits[-1]
            gap = float(lo[first_o] - lo[first_g])
        else:                                   # a draw: how close the drawn point lay to the edge of its bin
            gap = orc.first_margin
        assert gap < margin_thr, f"first token differs ({first_g} vs {first_o}) with margin {gap}"
        orc.x[-1] = int(first_g)
    return err


def lockstep_step(eng, orc, st: Stats, tol, margin_thr=2e-2, seq=0, stoch_margin=1e-3):
    return lockstep_step_batch(eng, [orc], [st], tol, margin_thr, stoch_margin)[0]


def lockstep_step_batch(eng, orcs, sts, tol, margin_thr=2e-2, stoch_margin=1e-3):
    """One step of every active slot; slot i is checked against orcs[i]."""
    all_toks = eng.draft_tree()
    for seq, (orc, st) in enumerate(zip(orcs, sts)):
        _check_draft(eng, orc, st, all_toks[seq], tol, margin_thr, seq)
    eng.verify()
    for seq, (orc, st) in enumerate(zip(orcs, sts)):
        _check_verify(eng, orc, st, tol, seq)
    out, lens, path = eng.accept()
    return [_check_accept(orc, st, out[seq], int(lens[seq]), path[seq], margin_thr, stoch_margin)
            for seq, (orc, st) in enumerate(zip(orcs, sts))]


def _check_draft(eng, orc, st, toks, tol, margin_thr, seq):
    d = orc.draft_tree(forced_tokens=toks)
    for (v, r, t_o, t_g, gap) in d["mismatches"]:
        assert gap < margin_thr, f"tree slot (node {v}, rank {r}): oracle {t_o} vs GPU {t_g}, score gap {gap}"
        st.excused_tree_slots += 1
    dl = eng.get_buffer(pkg.BUF_DRAFT_LOGITS, seq)
    df = eng.get_buffer(pkg.BUF_DRAFT_FEATURES, seq)
    for v, lo in orc.node_adj.items():
        st.max_draft_logit_err = max(st.max_draft_logit_err, float(np.abs(dl[v] - lo).max()))
        st.max_draft_feat_err = max(st.max_draft_feat_err, float(np.abs(df[v] - orc.node_f[v]).max()))
    assert st.max_draft_logit_err <= tol and st.max_draft_feat_err <= tol, \
        f"draft logits/features differ by {st.max_draft_logit_err} / {st.max_draft_feat_err}"


def _check_verify(eng, orc, st, tol, seq):
    F, L = orc.verify()
    st.max_logit_err = max(st.max_logit_err, float(np.abs(eng.get_buffer(pkg.BUF_LOGITS, seq) - L).max()))
    st.max_feat_err = max(st.max_feat_err, float(np.abs(eng.get_buffer(pkg.BUF_FEATURES, seq) - F).max()))
    assert st.max_logit_err <= tol and st.max_feat_err <= tol, \
        f"verify logits/features differ by {st.max_logit_err} / {st.max_feat_err}"


def _check_accept(orc, st, out, n, path, margin_thr, stoch_margin):
    g_path, g_out = [int(x) for x in path[:n]], [int(x) for x in out[:n]]
    r = orc.accept()
    assert 1 <= n <= orc.tree.D + 1
    assert g_path[0] == 0 and all(orc.tree.parent[g_path[i + 1]] == g_path[i] for i in range(n - 1))
    assert g_out[:-1] == [orc.tok[v] for v in g_path[1:]]
    if g_path != r["path"] or g_out != r["emitted"]:
        thr = margin_thr if orc.T == 0.0 else stoch_margin
        assert r["margin"] < thr, f"accept differs: GPU {g_path}/{g_out} oracle {r['path']}/{r['emitted']} margin {r['margin']}"
        st.excused_accepts += 1
    orc.commit(g_path, g_out[-1])
    st.steps += 1
    st.emitted += n
    st.lens.append(n)
    return g_out
