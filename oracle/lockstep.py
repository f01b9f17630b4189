"""Tolerance-validated lock-step comparison of an external decoder against the CPU oracle.

TEST INFRASTRUCTURE ONLY (part of the oracle package; imports nothing of the GPU library:
the other side's results arrive as plain numpy arrays).

Protocol.  Both sides consume the same attention bytes each step.  After each step the
other side's decisions are checked against the oracle's full ranking: every selected
(parent, token) must score within EPS of the oracle's Wb-th best or better, nothing better
than that by more than EPS may be missing, the order must agree up to EPS, every fused
score must agree within EPS.  Where the other side picked a different member of a near-tie
the oracle ADOPTS that decision and continues from it, so that later steps stay comparable;
the same holds for the threshold tests (ended-set entry, stop rules, end detection) and the
time indices (accepted if the oracle's forward variable at that frame is within EPS of its
maximum).  Anything outside EPS raises ParityError.  The report counts adopted decisions.
"""
import numpy as np

from . import OracleUtt, LOG0

EPS = 1e-4


class ParityError(AssertionError):
    pass


def _is0(v):
    return v < -1e29 or v == -np.inf


def _close(a, b, tol):
    if _is0(a) or _is0(b):
        return _is0(a) and _is0(b)
    return abs(a - b) <= tol


class Lockstep:
    def __init__(self, xs, cfg, eps=EPS, utt_ids=None):
        """xs: list of [T_i, V] fp32 posteriors; cfg: oracle.OrcCfg; utt_ids: their batch rows."""
        self.utts = [OracleUtt(x, cfg) for x in xs]
        self.ids = list(range(len(xs))) if utt_ids is None else list(utt_ids)
        self.cfg = cfg
        self.eps = eps
        self.B = cfg.beam
        self.report = dict(steps=0, adopted_sel=0, adopted_tau=0, adopted_eos=0, adopted_stop=0,
                           adopted_fin=0, max_score_err=0.0, max_ctc_err=0.0, exact_sel_steps=0,
                           utt_steps=0)

    def _fail(self, u, step, msg):
        raise ParityError(f"utt {u} step {step}: {msg}")

    def step(self, att, out, peek=None):
        """att: [U_all, Wb, V] fp32 (rows indexed by batch row); out: dict of numpy arrays
        parent, token, score, live, finished, tau, tau_end, eos_added, stopped (batch-indexed);
        peek: optional dict cand_id, cand_ctc, cand_joint, win_s, win_e, ctc_eos, joint_eos."""
        eps, B, rep = self.eps, self.B, self.report
        rep["steps"] += 1
        if self.cfg.win_union:
            # one window for the whole batch: needs every utterance of the batch in this check
            shares = [c for c in (o.union_contrib() for o in self.utts) if c is not None]
            if shares:
                tmin, emax = min(c[0] for c in shares), max(c[1] for c in shares)
                for o in self.utts:
                    o.set_union(tmin, emax)
        for o, u in zip(self.utts, self.ids):
            if o.finished:
                if not out["finished"][u]:
                    self._fail(u, o.step, "oracle finished earlier but the other side is still running")
                continue
            l = o.step + 1
            rep["utt_steps"] += 1
            o.score(att[u])
            live_old = np.array([o.hyp(j)["live"] for j in range(B)], bool)
            # ---- cell-level checks ------------------------------------------------------
            if peek is not None:
                s_o, e_o = o.windows()
                ids_o, ctc_o, J_o = o.cand_id(), o.cand_ctc(), o.cand_joint()
                ce_o, je_o = o.ctc_eos(), o.joint_eos()
                for j in range(B):
                    if not live_old[j]:
                        continue
                    if peek["win_s"][u, j] != s_o[j] or peek["win_e"][u, j] != e_o[j]:
                        self._fail(u, l, f"window of slot {j}: {peek['win_s'][u, j]},{peek['win_e'][u, j]} "
                                         f"vs oracle {s_o[j]},{e_o[j]}")
                    perm = np.argsort(peek["cand_id"][u, j], kind="stable")   # the other side's order is free
                    if not np.array_equal(peek["cand_id"][u, j][perm], ids_o[j]):
                        self._fail(u, l, f"candidate ids of slot {j} differ")
                    for i in range(o.K):
                        a, b = float(peek["cand_ctc"][u, j, perm[i]]), float(ctc_o[j, i])
                        if not _close(a, b, eps):
                            self._fail(u, l, f"ctc prefix score slot {j} cand {ids_o[j, i]}: {a} vs {b}")
                        if not _is0(b):
                            rep["max_ctc_err"] = max(rep["max_ctc_err"], abs(a - b))
                        a, b = float(peek["cand_joint"][u, j, perm[i]]), float(J_o[j, i])
                        if not _close(a, b, eps):
                            self._fail(u, l, f"joint score slot {j} cand {ids_o[j, i]}: {a} vs {b}")
                    for name, ref in (("ctc_eos", ce_o), ("joint_eos", je_o)):
                        a, b = float(peek[name][u, j]), float(ref[j])
                        if not _close(a, b, eps):
                            self._fail(u, l, f"{name} slot {j}: {a} vs {b}")
            # ---- eos-run stops -----------------------------------------------------------
            el, fire, margin = o.e2()
            stopped = np.zeros(B, np.int32)
            for j in range(B):
                if not live_old[j]:
                    continue
                g = int(out["stopped"][u, j])
                if g != int(fire[j]):
                    if el[j] and abs(margin[j]) <= eps:
                        rep["adopted_stop"] += 1
                    else:
                        self._fail(u, l, f"eos-run stop of slot {j}: {g} vs oracle {fire[j]} (margin {margin[j]})")
                stopped[j] = g
            # ---- selection ---------------------------------------------------------------
            o.rank(stopped)
            S = o.sorted_cands()
            n_exp = min(len(S), B)
            par, tok = out["parent"][u], out["token"][u]
            n_got = int((par >= 0).sum())
            if n_got != n_exp or not np.all(par[:n_got] >= 0):
                self._fail(u, l, f"new beam holds {n_got} hypotheses, oracle {n_exp}")
            lookup = {(int(c["parent"]), int(c["token"])): float(c["joint"]) for c in S}
            Jsel = []
            for n in range(n_got):
                key = (int(par[n]), int(tok[n]))
                if key not in lookup:
                    self._fail(u, l, f"selected {key} is not a finite candidate of the oracle")
                Jsel.append(lookup[key])
                err = abs(float(out["score"][u, n]) - lookup[key])
                rep["max_score_err"] = max(rep["max_score_err"], err)
                if err > eps:
                    self._fail(u, l, f"score of {key}: {out['score'][u, n]} vs {lookup[key]}")
            if len(set(zip(par[:n_got].tolist(), tok[:n_got].tolist()))) != n_got:
                self._fail(u, l, "a hypothesis was selected twice")
            if n_got:
                kth = float(S[n_exp - 1]["joint"])
                if min(Jsel) < kth - eps:
                    self._fail(u, l, f"selected score {min(Jsel)} below the oracle's Wb-th best {kth}")
                chosen = set(zip(par[:n_got].tolist(), tok[:n_got].tolist()))
                for c in S:
                    if float(c["joint"]) <= min(Jsel) + eps:
                        break
                    if (int(c["parent"]), int(c["token"])) not in chosen:
                        self._fail(u, l, f"candidate {(c['parent'], c['token'])} with score {c['joint']} "
                                         f"was left out (worst selected {min(Jsel)})")
                for n in range(n_got - 1):
                    if Jsel[n] < Jsel[n + 1] - eps:
                        self._fail(u, l, f"order of slots {n},{n + 1}: {Jsel[n]} < {Jsel[n + 1]}")
                same = (np.array_equal(par[:n_got], S["parent"][:n_got]) and
                        np.array_equal(tok[:n_got], S["token"][:n_got]))
                if same:
                    rep["exact_sel_steps"] += 1
                else:
                    rep["adopted_sel"] += 1
            else:
                rep["exact_sel_steps"] += 1
            # ---- ended-set entries -------------------------------------------------------
            forced = (l == o.lmax)
            best = o.best
            je = o.joint_eos()
            eos_add = np.zeros(B, np.int32)
            for j in range(B):
                if not live_old[j]:
                    continue
                own = bool(forced or stopped[j] or (je[j] > best))
                g = bool(out["eos_added"][u, j])
                if g != own:
                    if (not forced and not stopped[j] and np.isfinite(je[j]) and np.isfinite(best)
                            and abs(je[j] - best) <= eps):
                        rep["adopted_eos"] += 1
                    else:
                        self._fail(u, l, f"ended-set entry of slot {j}: {g} vs oracle {own} "
                                         f"(eos {je[j]}, best {best})")
                eos_add[j] = int(g)
            fin_own = o.commit(par[:n_got], tok[:n_got], eos_add, stopped)
            # ---- time indices ------------------------------------------------------------
            fin_g = bool(out["finished"][u])
            if not fin_g:
                mx_n, mx_b, lo = o.child_tau_info()
                s_o, e_o = o.windows()
                tau_over = np.full(B, -1, np.int32)
                tend_over = np.full(B, -1, np.int32)
                for n in range(n_got):
                    h = o.hyp(n)
                    e_win = e_o[par[n]]
                    for name, own, got, mx, which, over in (
                            ("tau", h["tau"], int(out["tau"][u, n]), mx_n[n], 0, tau_over),
                            ("tau_end", h["tau_end"], int(out["tau_end"][u, n]), mx_b[n], 1, tend_over)):
                        if got == own:
                            continue
                        ok = False
                        if lo[n] <= got <= e_win and np.isfinite(mx):
                            gam = o.hyp_gamma(n)[which]
                            ok = gam[got] >= mx - eps
                        if not ok:
                            self._fail(u, l, f"{name} of new slot {n}: {got} vs oracle {own}")
                        over[n] = got
                        rep["adopted_tau"] += 1
                if (tau_over >= 0).any() or (tend_over >= 0).any():
                    o.override(tau_over, tend_over, -1)
            # ---- finished flag -----------------------------------------------------------
            if fin_g != bool(fin_own):
                if o.e1_margin <= eps and not forced and n_got > 0:
                    o.override(None, None, int(fin_g))
                    rep["adopted_fin"] += 1
                else:
                    self._fail(u, l, f"finished flag {fin_g} vs oracle {bool(fin_own)} "
                                     f"(Eq. 4 margin {o.e1_margin})")
        return rep

    def all_finished(self):
        return all(o.finished for o in self.utts)

    def check_results(self, tokens, ntok, score, flags=None, frames=None):
        """Final hypotheses (batch-indexed arrays) against the oracle's ended-set argmax.  frames: the
        other side's time stamp (tau) of every label; the oracle's own are those it held when the labels
        were appended -- including every tau it adopted from the other side inside the tolerance during
        the steps -- so they must be equal."""
        for o, u in zip(self.utts, self.ids):
            lab, frm, sc, fb = o.result_frames()
            got = tokens[u, :ntok[u]]
            if not np.array_equal(got, lab):
                # a different member of a tie in the ended set is acceptable within EPS
                ties = [e for e in o.ended() if np.array_equal(got, e["labels"]) and _close(e["score"], sc, self.eps)]
                if ties:
                    self.report["adopted_fin"] += 1
                    if frames is not None and not any(np.array_equal(frames[u, :ntok[u]], e["taus"]) for e in ties):
                        raise ParityError(f"utt {u}: time stamps {frames[u, :ntok[u]].tolist()} of the tied result")
                    continue
                raise ParityError(f"utt {u}: final labels {got.tolist()} vs oracle {lab.tolist()}")
            if frames is not None and not np.array_equal(frames[u, :ntok[u]], frm):
                raise ParityError(f"utt {u}: time stamps {frames[u, :ntok[u]].tolist()} vs oracle {frm.tolist()}")
            if not _close(float(score[u]), sc if np.isfinite(sc) else LOG0, self.eps):
                raise ParityError(f"utt {u}: final score {score[u]} vs oracle {sc}")
            if flags is not None and bool(flags[u] & 1) != fb:
                raise ParityError(f"utt {u}: fallback flag {flags[u]} vs oracle {fb}")
