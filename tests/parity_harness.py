"""Drives GPU stages op by op, in lockstep with the oracle, and compares everything that is unique.

Order.  Every stage follows its own static op list; the global interleaving is the oracle
simulator's (any valid order gives the same numbers).  After each op on the oracle, the same op
runs on the GPU through the C ABI and its results are read back and compared.

What is unique.  Forward activations, losses, the op trace and the version ids are unique and
compared in full.  The ReLU derivative is a floating-point value deciding a 0/1: where a
pre-activation is within rounding of zero the two sides may legitimately decide differently
(their sums run in different orders and precisions).  Such elements are *detected* (stored
output positive on one side, zero on the other), required to be tiny on both sides and rare;
what they touch is treated apart: that minibatch's input-gradient rows are compared loosely;
in the update that consumes the minibatch, the weight/momentum rows of the units involved are
left out and the remaining rows (one of whose `minibatch` summands moved) get 2.5x the
tolerance.  Everything else must meet the tolerance.

Two modes.
  free    both sides run their own trajectory from the same initial state (fp32 mode, and
          short bf16 runs).  In bf16 the two trajectories separate step by step: one-ulp
          differences in re-rounded weights move pre-activations by ~1e-4, which flips ReLU
          decisions, which changes whole gradient rows -- inherent to the method's discrete
          decisions, not to either implementation.
  forced  after every update the GPU stage's latest version and momentum are overwritten
          with the oracle's (oracle -> GPU only), so every op is compared on the same
          weights; version/stash bookkeeping is still fully the GPU's own.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_1806_03377_amd as pd
from gpu_util import GpuStage, dev, empty_act, labels_dev, rel_err, to_dev, to_host
from oracle.pipeline import Stage
from oracle.schedule import OP_B, OP_F, OP_U, in_flight_depth, simulate, schedule_1f1b

TOL_F32 = 1e-4
TOL_BF16 = 2e-2
LOOSE = 10.0   # factor on the tolerance for input-gradient rows touched by an ambiguous ReLU decision
TOUCHED_UPDATE = 2.5   # factor for an update whose minibatch had a touched row (flagged units left out)


def _linears(layers):
    """The compute layers of a stage (everything but the loss) in the order the runtime numbers them: a
    branched block contributes its branch layers (branch 0 first) and then one entry for its concatenated output."""
    out = []
    for l in layers:
        if l[0] == "softmax_xent":
            continue
        if l[0] == "concat":
            for br in l[1]:
                out.extend(br)
            out.append(("concat_out",))
        else:
            out.append(l)
    return out


def _relu(L):
    return bool(L[3]) if L[0] == "linear" else (bool(L[8]) if L[0] == "conv2d" else False)


def _rows_of(L):
    """(units, weights per unit) of a parametrised layer: Linear (out, in); conv (c_out, kh*kw*c_in)."""
    if L[0] == "linear":
        return L[2], L[1]
    if L[0] == "conv2d":
        return L[2], L[3] * L[4] * L[1]
    return 0, 0


def _flat_keep(layers, units):
    """Boolean keep-mask over a stage's flat parameter vector, dropping the rows of flagged units."""
    parts = []
    for li, L in enumerate(_linears(layers)):
        if L[0] == "lstm":          # no ReLU, never flagged: keep everything
            parts.append(np.ones(4 * L[2] * (L[1] + L[2]) + 4 * L[2], dtype=bool))
            continue
        n_units, per = _rows_of(L)
        if not n_units:
            continue
        rows = np.ones(n_units, dtype=bool)
        if units.get(li):
            rows[sorted(units[li])] = False
        parts.append(np.repeat(rows, per))
        parts.append(rows.copy())
    return np.concatenate(parts)


def _global_order(S, noam, M, depth_override, vertical_sync=False):
    """(stage, Op) pairs in a valid global execution order."""
    if depth_override:
        assert S == 1
        return [(0, op) for op in schedule_1f1b(1, 1, M, 0, depth_override=depth_override)]
    ev = sorted(enumerate(simulate(S, noam, M)), key=lambda t: (t[1].start, t[0]))
    # simulate() already emits a valid order; sorting by start time keeps it valid (ties by emission)
    order = [(e.stage, e.op) for _, e in ev]
    if vertical_sync:   # same op order per stage; F and B carry the input stage's version (Section 3.4)
        lists = [schedule_1f1b(S, noam, M, s, vertical_sync=True) for s in range(S)]
        at = [0] * S
        for n, (s, op) in enumerate(order):
            vs = lists[s][at[s]]
            assert (vs.kind, vs.mb) == (op.kind, op.mb)
            order[n] = (s, vs)
            at[s] += 1
    return order


def run_case(stage_layers, params, xs, labs, *, noam, precision, depth_override=0, out_grads=None,
             lr=0.01, mu=0.9, mode="free", compare=True, verbose=False, in_hw=None, minibatch=None,
             force_acts=False, optimizer="sgd", eps=1.0, vertical_sync=False):
    """vertical_sync (Section 3.4): the version the input stage's forward pass read travels with the minibatch; every
    later stage is asked for that version of its own weights (pd_forward_versioned) and keeps as many versions as the
    input stage.

    force_acts (deep image stages): after every forward pass has been compared, the GPU stage's stored layer
    outputs -- and the next stage's input slot -- are overwritten with the oracle's (oracle -> GPU only).  In a
    deep bf16 chain one-ulp differences compound layer by layer into differing ReLU / max-pooling decisions; with
    the stored activations forced, every backward pass and update is compared on identical decisions and must
    meet the tolerance in full, while each forward pass is still the GPU's own from the stage input on."""
    bf16 = precision == pd.PD_BF16_F32ACC
    omode = "bf16" if bf16 else "f32"
    tol = TOL_BF16 if bf16 else TOL_F32
    S, M = len(stage_layers), len(xs)
    B = minibatch or xs[0].shape[0]     # (time-major sequence inputs are [T][B][I]: pass minibatch)
    has_loss = stage_layers[-1][-1][0] == "softmax_xent"
    depths = [depth_override or in_flight_depth(S, noam, s) for s in range(S)]
    order = _global_order(S, noam, M, depth_override, vertical_sync)
    os_ = [Stage(stage_layers[s], params[s], depths[s], omode, lr, mu, optimizer=optimizer, eps=eps,
                 ring_depth=depths[0] if vertical_sync else 0)
           for s in range(S)] if compare else None
    if compare:
        for o in os_:
            o.log = {}
    # in_hw: (h, w[, c]) of the input images of a single image stage, or one such tuple (or None) per stage
    hws = [in_hw] if (in_hw is None or not isinstance(in_hw[0], (tuple, list, type(None)))) else list(in_hw)
    if len(hws) == 1 and S > 1:
        assert in_hw is None, "give one input size per stage"
        hws = [None] * S
    gs = [GpuStage(stage_layers[s], params[s], minibatch=B, precision=precision, stage_index=s, num_stages=S,
                   noam=noam, in_flight_override=depth_override, lr=lr, momentum=mu, in_hw=hws[s],
                   optimizer=1 if optimizer == "rmsprop" else 0, eps=eps, vertical_sync=vertical_sync)
          for s in range(S)]
    rings = [pd.pd_stage_ring_depth(g.h) for g in gs]
    tag = {}           # vertical sync: minibatch -> version read by the input stage's forward pass
    keep = []          # device tensors that must outlive the enqueued work
    losses = torch.zeros(M, dtype=torch.float32, device=dev())
    o_losses = [None] * M
    o_act, o_grad, o_act_size = {}, {}, {}
    touched = {i: set() for i in range(M)}      # rows of minibatch i touched by an ambiguous decision so far
    flips_at, units_at = {}, {}
    n_flips = n_elems = n_strict = n_updates = 0
    try:
        for s, op in order:
            g, mb = gs[s], op.mb
            o = os_[s] if compare else None
            lin = _linears(stage_layers[s])
            if op.kind == OP_F:
                # ---- oracle ----
                if compare:
                    xin = np.asarray(xs[mb], dtype=np.float64) if s == 0 else o_act.pop((mb, s - 1))
                    y_o, loss_o = o.forward(mb, xin, labs[mb] if (s == S - 1 and has_loss) else None,
                                            version=tag[mb] if (vertical_sync and s > 0) else None)
                    if s == S - 1:
                        o_losses[mb] = loss_o
                    else:
                        o_act[(mb, s)] = y_o
                        o_act_size[s + 1] = y_o.size // B
                # ---- GPU ----
                if vertical_sync:
                    if s == 0:
                        tag[mb] = pd.pd_stage_version(g.h)
                    assert tag[mb] == op.version
                else:
                    assert pd.pd_stage_version(g.h) == op.version
                if s == 0:
                    x = to_dev(xs[mb], bf16); keep.append(x); xptr = x.data_ptr()
                else:
                    xptr = pd.pd_stage_input_slot(g.h, mb)
                yptr = pd.pd_stage_input_slot(gs[s + 1].h, mb) if s < S - 1 else 0
                lab = 0
                if s == S - 1 and has_loss:
                    l_t = labels_dev(labs[mb]); keep.append(l_t); lab = l_t.data_ptr()
                pd.pd_forward_versioned(g.h, mb, tag[mb] if vertical_sync else -1, xptr, lab, yptr,
                                        losses[mb:].data_ptr() if lab else 0)
                assert pd.pd_stage_version(g.h, mb) == op.version
                if not compare:
                    continue
                assert o.trace[-1] == (OP_F, mb, op.version, op.slot)
                acts_o = o.log[mb]["acts"]
                flat_o = o.log[mb]["flat"]
                rows, units = set(), {}
                for li, L in enumerate(lin):
                    y_o = flat_o[li].reshape(B, -1)
                    y_g = pd.pd_stage_debug_read(g.h, 0, mb, li, y_o.shape).astype(np.float64)
                    assert rel_err(y_g, y_o) <= tol, ("forward", s, mb, li, rel_err(y_g, y_o))
                    if _relu(L):
                        diff = (y_g > 0) != (y_o > 0)
                        n_elems += diff.size
                        if diff.any():
                            n_flips += int(diff.sum())
                            lim = tol * np.abs(y_o).max()
                            assert np.all(np.abs(y_g[diff]) <= lim) and np.all(np.abs(y_o[diff]) <= lim)
                            rows |= set(np.nonzero(diff)[0].tolist())
                            n_units = _rows_of(L)[0]          # conv: the unit is the output channel
                            units[li] = set((np.nonzero(diff)[1] % n_units).tolist())
                flips_at[(s, mb)] = rows
                units_at[(s, mb)] = units
                if s < S - 1:   # the hand-off: the next stage's input slot holds exactly this output
                    shp = acts_o[-1].reshape(B, -1).shape
                    nxt = pd.pd_stage_debug_read(gs[s + 1].h, 1, mb, 0, shp)
                    assert np.array_equal(nxt, pd.pd_stage_debug_read(g.h, 0, mb, len(lin) - 1, shp))
                if force_acts:
                    for li, L in enumerate(lin):
                        if L[0] != "lstm":
                            pd.pd_stage_debug_write(g.h, 0, mb, li, flat_o[li])
                    if s < S - 1:
                        pd.pd_stage_debug_write(gs[s + 1].h, 1, mb, 0, flat_o[-1])
                    flips_at[(s, mb)], units_at[(s, mb)] = set(), {}     # decisions are now the oracle's on both sides
                if verbose:
                    print(f"F stage {s} mb {mb} v{op.version}: rows with ambiguous ReLU decisions {len(rows)} "
                          f"(total elements {n_flips}/{n_elems})", flush=True)
            elif op.kind == OP_B:
                if s == 0:
                    n_in = int(np.asarray(xs[0]).size // B)
                elif lin[0][0] == "linear":
                    n_in = lin[0][1]
                elif hws[s] is not None and len(hws[s]) == 3:
                    n_in = int(np.prod(hws[s]))
                else:
                    n_in = int(o_act_size[s])
                if compare:
                    if s == S - 1:
                        dy_o = None if has_loss else np.asarray(out_grads[mb], dtype=np.float64)
                    else:
                        dy_o = o_grad.pop((mb, s + 1))
                    dx_o = o.backward(mb, dy_o, need_dx=True)
                    if s > 0:
                        o_grad[(mb, s)] = dx_o
                    dx_o = dx_o.reshape(B, -1)
                assert pd.pd_stage_version(g.h, mb) == op.version
                if s == S - 1:
                    dyptr = 0
                    if not has_loss:
                        dy = to_dev(out_grads[mb], bf16); keep.append(dy); dyptr = dy.data_ptr()
                else:
                    dyptr = pd.pd_stage_grad_slot(g.h, mb)
                if s > 0:
                    dxptr, dx_t = pd.pd_stage_grad_slot(gs[s - 1].h, mb), None
                else:
                    dx_t = empty_act(B, n_in, bf16); keep.append(dx_t); dxptr = dx_t.data_ptr()
                pd.pd_backward(g.h, mb, dyptr, dxptr)
                if not compare:
                    continue
                assert o.trace[-1] == (OP_B, mb, op.version, op.slot)
                if s > 0:
                    dx_g = pd.pd_stage_debug_read(gs[s - 1].h, 2, mb, 0, (B, n_in)).astype(np.float64)
                else:
                    torch.cuda.synchronize()
                    dx_g = to_host(dx_t)
                touched[mb] |= flips_at[(s, mb)]
                ok = np.array([m not in touched[mb] for m in range(B)])
                scale = max(float(np.abs(dx_o).max()), 1e-30)
                err_all = float(np.max(np.abs(dx_g - dx_o))) / scale
                err = float(np.max(np.abs(dx_g[ok] - dx_o[ok]))) / scale if ok.any() else 0.0
                if verbose:
                    print(f"B stage {s} mb {mb}: rows at full tolerance {int(ok.sum())}/{B}, err {err:.3e} "
                          f"(all rows {err_all:.3e})", flush=True)
                assert err <= tol, ("backward", s, mb, err)
                assert err_all <= LOOSE * tol, ("backward, rows touched by ambiguous decisions", s, mb, err_all)
            else:
                if compare:
                    o.update(mb)
                pd.pd_update(g.h)
                assert pd.pd_stage_version(g.h) == op.version
                if not compare:
                    continue
                assert o.trace[-1] == (OP_U, mb, op.version, op.slot)
                if mode == "forced" or op.version == M:
                    # compare what this update produced (forced: every update; free: the final state)
                    strict = not touched[mb] or mode == "free"
                    t = tol if strict else TOUCHED_UPDATE * tol
                    k = slice(None) if strict else _flat_keep(stage_layers[s], units_at[(s, mb)])
                    n_updates += 1
                    n_strict += int(strict)
                    p = pd.pd_stage_get_params(g.h); m = pd.pd_stage_get_momentum(g.h)
                    ring = pd.pd_stage_get_params(g.h, -1, True)
                    for name, got, ref in (("master", p, o.master), ("momentum", m, o.mom), ("ring", ring, o.versions[-1])):
                        e = float(np.max(np.abs(got[k] - ref[k]))) / max(float(np.abs(ref).max()), 1e-30)
                        if verbose:
                            print(f"U stage {s} mb {mb} -> v{op.version}: {name} err {e:.3e} (limit {t:.1e})", flush=True)
                        assert e <= t, (name, s, mb, e)
                    if rings[s] >= 2 and op.version >= 1:   # an older version still held by the ring
                        old = pd.pd_stage_get_params(g.h, op.version - 1, True)
                        assert rel_err(old, o.versions[op.version - 1]) <= t, ("ring history", s, mb)
                if mode == "forced":
                    pd.pd_stage_overwrite_latest(g.h, o.master.astype(np.float32), o.mom.astype(np.float32))
        torch.cuda.synchronize()
        out = {"losses": to_host(losses), "params": [pd.pd_stage_get_params(g.h) for g in gs],
               "mom": [pd.pd_stage_get_momentum(g.h) for g in gs], "flips": n_flips,
               "trace": [pd.pd_stage_trace(g.h) for g in gs]}
        if compare:
            assert n_flips <= max(2, 1e-3 * n_elems), (n_flips, n_elems)
            out["updates_compared"] = (n_strict, n_updates)
            if has_loss:
                for i in range(M):
                    assert abs(out["losses"][i] - o_losses[i]) <= tol * abs(o_losses[i]), ("loss", i)
            for s in range(S):
                assert out["trace"][s] == [tuple(t) for t in os_[s].trace], ("trace", s)
                assert os_[s].latest == M and not os_[s].stash
        return out
    finally:
        for g in gs:
            g.close()
