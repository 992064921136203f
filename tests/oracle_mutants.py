"""Planted mistakes for the oracle's bf16 rounding points (test infrastructure, CPU only).

Each entry replaces one piece of the source text of one oracle function: a `store()` removed, or one added where the
numerics contract keeps a value in float.  `make_mutant` compiles the changed function in a copy of the oracle's
namespace; a test installs it with monkeypatch and expects a pin to fail, or a crafted case to change its result."""
import inspect

from oracle import ee_oracle as O

_NORM = 'rmsnorm(h, m.weights["layers"][i - 1]["{g}"], m.rms_eps)'
_DEFERRED = '(store(h * m.weights["layers"][i - 1]["{g}"].to(F64), dt) / torch.sqrt((h * h).mean(dim=-1, keepdim=True) + m.rms_eps))'

MUTANTS = {
    # name: (oracle function, text to replace, replacement, which occurrence)
    "attention output not rounded": ("layer_forward", "a = store(a.reshape(B, H * dh), dt)", "a = a.reshape(B, H * dh)", 0),
    "SwiGLU product not rounded": ("layer_forward", "act = store(g / (1.0 + torch.exp(-g)) * u, dt)",
                                   "act = g / (1.0 + torch.exp(-g)) * u", 0),
    "FFN-norm operand not rounded": ("layer_forward", "x = store(" + _NORM.format(g="g_ffn") + ", dt)",
                                     "x = " + _NORM.format(g="g_ffn"), 0),
    "attention-norm operand not rounded": ("layer_forward", "x = store(" + _NORM.format(g="g_attn") + ", dt)",
                                           "x = " + _NORM.format(g="g_attn"), 0),
    "residual stream rounded after the FFN": ("layer_forward", 'return h + act @ _w(m, i, "w_down").T',
                                              'return store(h + act @ _w(m, i, "w_down").T, dt)', 0),
    "residual stream rounded after attention": ("layer_forward", 'h = h + a @ _w(m, i, "w_o").T',
                                                'h = store(h + a @ _w(m, i, "w_o").T, dt)', 0),
    "q rounded": ("layer_forward", "q = rope(q, pos, m.rope_theta)", "q = store(rope(q, pos, m.rope_theta), dt)", 0),
    "gate rounded before the product": ("layer_forward", 'g = x @ _w(m, i, "w_gate").T', 'g = store(x @ _w(m, i, "w_gate").T, dt)', 0),
    # the row factor of RMSNorm applied after the rounding instead of before it (what a kernel does that folds the
    # factor into the consuming projection)
    "FFN-norm row factor applied after the rounding": ("layer_forward", "x = store(" + _NORM.format(g="g_ffn") + ", dt)",
                                                       "x = " + _DEFERRED.format(g="g_ffn"), 0),
    "attention-norm row factor applied after the rounding": ("layer_forward", "x = store(" + _NORM.format(g="g_attn") + ", dt)",
                                                             "x = " + _DEFERRED.format(g="g_attn"), 0),
    "exit-head operand not rounded": ("head_logits", 'x = store(rmsnorm(h, m.weights["g_final"], m.rms_eps), m.dtype)',
                                      'x = rmsnorm(h, m.weights["g_final"], m.rms_eps)', 0),
    "exit-head logits rounded": ("head_logits", 'return x @ m.weights["w_lm"].to(F64).T',
                                 'return store(x @ m.weights["w_lm"].to(F64).T, m.dtype)', 0),
    "filling operand not rounded": ("kv_fill", "x = store(" + _NORM.format(g="g_attn") + ", dt)",
                                    "x = " + _NORM.format(g="g_attn"), 0),
    "filled K rounded before the rotation": ("kv_fill", 'k = rope((x @ _w(m, i, "w_k").T).reshape(B, H, dh), pos, m.rope_theta)',
                                             'k = rope(store(x @ _w(m, i, "w_k").T, dt).reshape(B, H, dh), pos, m.rope_theta)', 0),
}


def make_mutant(fn_name, old, new, which=0):
    """The oracle function `fn_name` with one piece of its source text replaced."""
    src = inspect.getsource(getattr(O, fn_name))
    assert src.count(old) > which, f"the oracle's source no longer contains {old!r}"
    parts = src.split(old)
    src = old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])
    ns = dict(vars(O))
    exec(compile(src, f"<mutant of {fn_name}>", "exec"), ns)
    return ns[fn_name]


class planted:
    """Context manager: the oracle with the named mistake planted."""

    def __init__(self, name):
        self.fn_name, old, new, which = MUTANTS[name]
        self.mutant = make_mutant(self.fn_name, old, new, which)

    def __enter__(self):
        self.saved = getattr(O, self.fn_name)
        setattr(O, self.fn_name, self.mutant)
        return self

    def __exit__(self, *exc):
        setattr(O, self.fn_name, self.saved)
        return False
