"""Are the oracle's pins sharp?  Plausible mistakes are planted in the oracle, one at a time and on the
CPU only -- a dropped term, a wrong sign, an index off by one, a transposed operand, a wrong head
mapping -- and for every one of them at least one pin of tests/test_oracle_pins.py or
tests/test_oracle_scheduling.py has to fail.  A mistake that every pin lets through would mean the
oracle could be wrong in that way without anybody noticing.

A mistake is planted by re-compiling one function of the oracle module from its own source text with
one expression replaced; the original function is put back afterwards.
"""
import inspect
import textwrap

import pytest

from oracle import paged_attention as O
from oracle import scheduling as S

import test_oracle_pins as attention_pins
import test_oracle_scheduling as scheduling_pins


def pin_calls(module):
    """Every test function of a pin module, once per parameter set: (name, callable without arguments)."""
    calls = []
    for name, fn in sorted(vars(module).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        sets = [{}]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name != "parametrize":
                continue
            names = [n.strip() for n in mark.args[0].split(",")]
            grown = []
            for values in mark.args[1]:
                if len(names) == 1:
                    values = (values,)
                grown += [dict(s, **dict(zip(names, values))) for s in sets]
            sets = grown
        for kw in sets:
            wanted = set(inspect.signature(fn).parameters)
            if not set(kw) >= wanted - {"tmp_path"} or "tmp_path" in wanted:
                continue
            calls.append((f"{name}{kw or ''}", lambda fn=fn, kw=kw: fn(**kw)))
    return calls


class planted:
    """Context manager: module.function re-compiled with `old` replaced by `new` in its source."""

    def __init__(self, module, function, old, new):
        self.module, self.function = module, function
        self.original = getattr(module, function)
        src = textwrap.dedent(inspect.getsource(self.original))
        assert src.count(old) == 1, f"{function}: expected exactly one {old!r} in the source"
        self.src = src.replace(old, new)

    def __enter__(self):
        scope = self.module.__dict__
        exec(compile(self.src, f"<{self.function} with a planted mistake>", "exec"), scope)
        assert getattr(self.module, self.function) is not self.original

    def __exit__(self, *exc):
        setattr(self.module, self.function, self.original)
        return False


def first_pin_that_fails(calls):
    for name, call in calls:
        try:
            call()
        except Exception:            # an assertion, or the mistake made the oracle raise
            return name
    return None


ATTENTION_MISTAKES = [
    # --- the arithmetic of softmax attention
    ("scale dropped",                   "attention_rows", "z = scale * (q @ K[:L].T)", "z = (q @ K[:L].T)"),
    ("sign of the scores",              "attention_rows", "z = scale * (q @ K[:L].T)", "z = -scale * (q @ K[:L].T)"),
    ("scores taken from V",             "attention_rows", "(q @ K[:L].T)", "(q @ V[:L].T)"),
    ("values taken from K",             "attention_rows", "o = (w @ V[:L]) / l", "o = (w @ K[:L]) / l"),
    ("one hidden key visible",          "attention_rows", "np.arange(L)[None, :] >= nv[:, None]", "np.arange(L)[None, :] > nv[:, None]"),
    ("weights not normalised",          "attention_rows", "o = (w @ V[:L]) / l", "o = (w @ V[:L])"),
    ("normalised by the largest weight", "attention_rows", "l = w.sum(axis=1, keepdims=True)", "l = w.max(axis=1, keepdims=True)"),
    ("exp of the scores' negative",     "attention_rows", "w = np.exp(z - m)", "w = np.exp(m - z)"),
    # --- which keys a row sees
    ("decode leaves out its own token", "paged_decode", "scale, [L] * G)", "scale, [L - 1 if L > 1 else L] * G)"),
    ("causal diagonal left out",        "paged_prefill_chunk", "vis = [p + r + 1 for r in rows]", "vis = [max(p + r, 1) for r in rows]"),
    ("prior tokens forgotten",          "paged_prefill_chunk", "vis = [p + r + 1 for r in rows]", "vis = [r + 1 for r in rows]"),
    ("chunk sees its whole self",       "paged_prefill_chunk", "vis = [p + r + 1 for r in rows]", "vis = [p + max(rows) + 1 for r in rows]"),
    # --- heads
    ("query heads interleaved over kv heads", "paged_decode", "attention_rows(q64[s, kvh * G:(kvh + 1) * G]", "attention_rows(q64[s, kvh::pool.Hkv]"),
    ("prefill head mapping h % Hkv",    "paged_prefill_chunk", "h = kvh * G + g", "h = g * pool.Hkv + kvh"),
    # --- paging and layout
    ("range boundary off by one",       "resolve_block", "if block < first + n:", "if block <= first + n:"),
    ("block index inside a range not rebased", "resolve_block", "return r, block - first", "return r, block"),
    ("slot taken from the block index", "token_slot", "t % B", "t // B % B"),
    ("table indexed by token",          "token_slot", "table_row[t // B]", "table_row[min(t, len(table_row) - 1) // max(B // 2, 1)]"),
    ("K rows of a page not strided by head_dim", "k_elem_offset", "(slot % T) * pool.d", "(slot % T)"),
    ("V stored [token][dim]",           "v_elem_offset", "T * pool.d + j * T + slot % T", "T * pool.d + (slot % T) * pool.d + j"),
    ("V read in front of K",            "v_elem_offset", "(slot // T) * 2 * T * pool.d + T * pool.d", "(slot // T) * 2 * T * pool.d"),
    ("pages of a block not per kv head", "k_elem_offset", "(local_block * pool.Hkv + kvh)", "(local_block * pool.Hkv)"),
    ("tile of 64 tokens not split in four", "tile_tokens", "return min(B, TILE_TOKENS)", "return B"),
    ("V gathered without the transpose", "gather_kv", "V[b0:b0 + n] = vt[:, :n].T", "V[b0:b0 + n] = vt.reshape(T, d)[:n]"),
    # --- element formats
    ("bf16 widened as the low half",    "widen", "<< np.uint32(16)", "<< np.uint32(0)"),
    ("E4M3 exponent bias 8",            "widen", "(e - 7).astype(np.int64)", "(e - 8).astype(np.int64)"),
    ("E4M3 subnormals scaled like normals", "widen", "np.ldexp(m / 8.0, -6)", "np.ldexp(m / 8.0, -7)"),
    ("E4M3 sign ignored",               "widen", "np.where((c >> 7) & 1, -1.0, 1.0)", "np.where((c >> 7) & 0, -1.0, 1.0)"),
    # --- merge of split-K partial results
    ("merge factors inverted",          "merge_partials", "f = np.exp(m - M)", "f = np.exp(M - m)"),
    ("merge sums l without its factor", "merge_partials", "(f * l).sum()", "l.sum()"),
    # --- append
    ("append writes V like K",          "kv_append", "mem[v_elem_offset(pool, local, kvh, slot, j)] = v_new[i, kvh, j]",
     "mem[v_elem_offset(pool, local, kvh, slot, 0) + j] = v_new[i, kvh, j]"),
    ("append ignores the token's position", "kv_append", "int(pos_of_tok[i]), pool.B)", "i, pool.B)"),
]

SCHEDULING_MISTAKES = [
    ("Eq. 1 without the diagonal",      "attention_pairs", "(c * c + c) // 2", "(c * c) // 2"),
    ("Eq. 1 without the prefix term",   "attention_pairs", "p * c + ", "0 * p * c + "),
    ("Eq. 1: per-token term dropped",   "chunk_cost", "+ beta * c", "+ 0 * beta * c"),
    ("Eq. 3: gamma charged per chunk",  "microbatch_cost", "- (len(live) - 1) * gamma", "- 0 * gamma"),
    ("Eq. 3: gamma never charged",      "microbatch_cost", "- (len(live) - 1) * gamma", "- len(live) * gamma"),
    ("a cut request restarts at its old prior", "split_microbatch", "(r, p + k, c - k)", "(r, p, c - k)"),
    ("split keeps the first balanced cut it meets, worst first", "split_microbatch", "d < best[0]", "d > best[0]"),
    ("lookahead ignores the token threshold on the right half", "lookahead",
     "tokens_of(l) >= min_tokens and tokens_of(r) >= min_tokens", "tokens_of(l) >= min_tokens"),
    ("Algorithm 1 merges the two LARGEST groups", "drop_plan", "heap = [(len(g), order, g)", "heap = [(-len(g), order, g)"),
    ("Algorithm 1: a merge frees one layer, not one copy", "drop_plan", "freed += copy_bytes", "freed += layer_bytes"),
    ("pipeline stages overlap by one layer", "stage_layers", "((j + 1) * L) // g", "min(((j + 1) * L) // g + 1, L)"),
]


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("what,function,old,new", ATTENTION_MISTAKES, ids=[m[0] for m in ATTENTION_MISTAKES])
def test_a_mistake_planted_in_the_attention_oracle_fails_a_pin(what, function, old, new):
    calls = pin_calls(attention_pins)
    assert len(calls) >= 20
    with planted(O, function, old, new):
        caught_by = first_pin_that_fails(calls)
    assert caught_by is not None, f"no pin notices: {what}"
    assert first_pin_that_fails([c for c in calls if c[0] == caught_by]) is None, "the pin fails without the mistake too"


@pytest.mark.parametrize("what,function,old,new", SCHEDULING_MISTAKES, ids=[m[0] for m in SCHEDULING_MISTAKES])
def test_a_mistake_planted_in_the_scheduling_oracle_fails_a_pin(what, function, old, new):
    calls = pin_calls(scheduling_pins)
    assert len(calls) >= 10
    with planted(S, function, old, new):
        caught_by = first_pin_that_fails(calls)
    assert caught_by is not None, f"no pin notices: {what}"
    assert first_pin_that_fails([c for c in calls if c[0] == caught_by]) is None, "the pin fails without the mistake too"


def test_recompiling_the_functions_unchanged_fails_no_pin():
    """The planting itself is harmless: every function named above, re-compiled from its unchanged source,
    still passes every pin (so a pin that fails above fails because of the mistake)."""
    for module, mistakes, pins in ((O, ATTENTION_MISTAKES, attention_pins), (S, SCHEDULING_MISTAKES, scheduling_pins)):
        calls = pin_calls(pins)
        for function, old in sorted({(m[1], m[2]) for m in mistakes}):
            with planted(module, function, old, old):
                assert first_pin_that_fails(calls) is None, function
