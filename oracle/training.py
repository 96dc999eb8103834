"""Oracle composition of one iteration of encrypted logistic-regression training with Nesterov momentum and
Bootstrap (test infrastructure only): gradient step (oracle/classifier.py), look-ahead update
W' = (1 + gamma) V' - gamma V, division by about 2^shrink_bits with one rescale, Bootstrap with the gain that returns
to the working scale (oracle/bootstrap.py)."""
from . import bootstrap as ob
from . import classifier as oc


def _const(o, v, s, level):
    iv = int(round(v * s))
    return [iv % o.q[i] for i in range(level)]


def iterate(o, X, W, V, Y, keys, plan, block, scale, lr, gamma, n_samples, a=None, pts_cts=None, pts_stc=None,
            shrink_bits=6, c15=None):
    """W at level plan.out_level, V at plan.out_level - 8 (or above), X at plan.out_level; all at `scale`.
    Returns (W_next, V_next)."""
    level = plan.out_level
    q = [float(v) for v in o.q]
    v_new = oc.train_step(o, X, W, Y, keys["relin"], keys["rot"], level, scale, lr, n_samples, a, block, c15)
    shrink = int(round(o.q[1] / 2.0**shrink_bits))
    delta_in = scale * shrink / q[1]
    gain = scale / (delta_in * plan.natural_factor(o))
    w_next = []
    for vn, vo in zip(v_new, V):
        lv = vn.shape[1]
        up = o.cmult(vn, _const(o, 1.0 + gamma, q[lv - 1], lv))
        down = o.cmult(o.moddrop(vo, lv), _const(o, gamma, q[lv - 1], lv))
        w = o.rescale(o.sub(up, down))
        small = o.rescale(o.cmult(o.moddrop(w, 2), [shrink % o.q[0], shrink % o.q[1]]))
        out, lvl, _ = ob.bootstrap(o, small, keys, plan, pts_cts, pts_stc, gain)
        assert lvl == level
        w_next.append(out)
    return w_next, v_new
