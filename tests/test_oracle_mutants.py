"""Do the pins hold the oracle?  Plausible mistakes are planted in the oracle's source (on the CPU,
in a copy of the module that only this test sees) and the pin tests are run against each: every
planted mistake -- a dropped term, a wrong sign or index, a swapped step, an off-by-one -- must make
at least one pin fail.  The unaltered source must pass them all, run the same way.

A mistake is a textual replacement that must match the oracle's source exactly once, so this
file fails loudly, instead of silently testing nothing, when the oracle's text changes.
"""
import importlib.util
import inspect
import itertools
import os
import sys
import types

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

ALLOC_PINS = ["test_oracle_alloc.py", "test_oracle_eviction.py"]
EVICT_PINS = ["test_oracle_eviction.py", "test_oracle_alloc.py"]      # the same pins, the likelier ones first
ATTN_PINS = ["test_oracle_attn.py"]

# (name, oracle module, [(text, replacement)], pin files)
MUTANTS = [
    # ---- Sec. 1 / 4.1: compatible page size, small-page size
    ("lcm is the product", "alloc", [("out = out * s // math.gcd(out, s)", "out = out * s")], ALLOC_PINS),
    ("lcm is the largest size", "alloc", [("out = out * s // math.gcd(out, s)", "out = max(out, s)")], ALLOC_PINS),
    ("small page holds K only", "alloc", [("per_token_per_layer = 2 * n_kv_heads * head_dim * elem_bytes",
                                          "per_token_per_layer = n_kv_heads * head_dim * elem_bytes")], ALLOC_PINS),
    ("small page holds one layer", "alloc", [("return per_token_per_layer * n_layers * tokens_per_page",
                                             "return per_token_per_layer * tokens_per_page")], ALLOC_PINS),
    ("small pages per large page off by one", "alloc", [("self.r = [self.large_bytes // s for s in self.S]",
                                                        "self.r = [self.large_bytes // s + 1 for s in self.S]")], ALLOC_PINS),
    ("byte offset in units of the large page", "alloc", [("return sid * self.S[k]", "return sid * self.large_bytes")], ALLOC_PINS),
    # ---- Sec. 4.3: the three steps
    ("step 1 ignores the request", "alloc", [("mine = self._larges_with_room(k, self.large_req == request)",
                                             "mine = self._larges_with_room(k, everyone)")], ALLOC_PINS),
    ("step 1 looks at other requests' pages", "alloc", [("mine = self._larges_with_room(k, self.large_req == request)",
                                                        "mine = self._larges_with_room(k, self.large_req != request)")], ALLOC_PINS),
    ("new large page not tied to the request", "alloc", [("            self.large_kind[large] = k\n            self.large_req[large] = request\n            return self._take_lowest_free_slot(k, large)",
                                                         "            self.large_kind[large] = k\n            return self._take_lowest_free_slot(k, large)")], ALLOC_PINS),
    ("highest free slot instead of lowest", "alloc", [("slot = int(np.flatnonzero(slots == 0)[0])", "slot = int(np.flatnonzero(slots == 0)[-1])")], ALLOC_PINS),
    ("last free large page instead of first", "alloc", [("            large = int(free_large[0])\n            self.large_kind[large] = k\n            self.large_req[large] = request\n            return self._take_lowest_free_slot(k, large)",
                                                        "            large = int(free_large[-1])\n            self.large_kind[large] = k\n            self.large_req[large] = request\n            return self._take_lowest_free_slot(k, large)")], ALLOC_PINS),
    ("a type may take slots of another type's large page", "alloc", [("return np.flatnonzero(mask & (self.large_kind == k) & unused)",
                                                                      "return np.flatnonzero(mask & (self.large_kind >= 0) & unused)")], ALLOC_PINS),
    ("large page never returned", "alloc", [("        if not self._slots(k, large).any():          # every small page unused\n            self.large_kind[large] = -1",
                                            "        if False:\n            self.large_kind[large] = -1")], ALLOC_PINS),
    ("large page returned while one page is used", "alloc", [("if not self._slots(k, large).any():          # every small page unused",
                                                             "if not self._slots(k, large).all():")], ALLOC_PINS),
    ("free ignores the reference count", "alloc", [("        self.refcount[k][sid] -= 1\n        large = sid // self.r[k]",
                                                   "        self.refcount[k][sid] = 0\n        large = sid // self.r[k]")], ALLOC_PINS),
    # ---- Sec. 5.1: the window's need set
    ("window one token short", "alloc", [("return max(0, seq_len - window)", "return max(0, seq_len - window + 1)")], ALLOC_PINS),
    ("window one token long", "alloc", [("return max(0, seq_len - window)", "return max(0, seq_len - window - 1)")], ALLOC_PINS),
    ("page freed while its last token is needed", "alloc", [("if T * (p + 1) <= lo and lst[p] >= 0:", "if T * p <= lo and lst[p] >= 0:")], ALLOC_PINS),
    ("page kept one token too long", "alloc", [("if T * (p + 1) <= lo and lst[p] >= 0:", "if T * (p + 1) < lo and lst[p] >= 0:")], ALLOC_PINS),
    ("pages counted with floor", "alloc", [("need = -(-new_len // T)", "need = new_len // T")], ALLOC_PINS),
    ("shared page not counted", "alloc", [("                self.pool.ref(k, s[p])\n", "                pass\n")], ALLOC_PINS),
    # ---- Sec. 5.4: states, five steps, LRU
    ("released page always empty", "alloc", [("self.cached[k][sid] = bool(keep_cached)", "self.cached[k][sid] = False")], EVICT_PINS),
    ("large page evictable when any small page is", "alloc", [("if not self.cached[ko][ids].all():       # evictable = every small page evictable",
                                                              "if not self.cached[ko][ids].any() or self.refcount[ko][ids].any():")], EVICT_PINS),
    ("large page's time is its earliest access", "alloc", [("key = (int(self.last_access[ko][ids].max()),", "key = (int(self.last_access[ko][ids].min()),")], EVICT_PINS),
    ("most recently used large page evicted", "alloc", [("if best_key is None or key < best_key:", "if best_key is None or key > best_key:")], EVICT_PINS),
    ("most recently used small page evicted", "alloc", [("sid = min(keys)[2]", "sid = max(keys)[2]")], EVICT_PINS),
    ("shorter prefix evicted first among equal times", "alloc", [("keys = [(int(self.last_access[k][s]), -int(self.prefix_length[k][s]), int(s)) for s in cand]",
                                                                 "keys = [(int(self.last_access[k][s]), int(self.prefix_length[k][s]), int(s)) for s in cand]")], EVICT_PINS),
    ("steps 3 and 4 swapped", "alloc", [("        if best is not None:\n", "        anyone4 = self._larges_with_empty(k, np.ones(self.n_large, dtype=bool))\n        if anyone4.size:\n            return self._take_lowest_empty(k, int(anyone4[0])), []\n        if best is not None:\n")], EVICT_PINS),
    ("evicted large page keeps its old type", "alloc", [("            self.large_kind[best] = k            # all its small pages are empty now: re-typed\n", "")], EVICT_PINS),
    ("eviction not reported", "alloc", [("return self._take_lowest_empty(k, best), evicted", "return self._take_lowest_empty(k, best), []")], EVICT_PINS),
    ("cached large page returned as free", "alloc", [("if not self.refcount[k][sl].any() and not self.cached[k][sl].any():", "if not self.refcount[k][sl].any():")], EVICT_PINS),
    ("finished request keeps its pages", "alloc", [("                if sid >= 0:\n                    self.pool.free(k, sid)\n", "                pass\n")], EVICT_PINS),
    ("finished request frees the first kind only", "alloc", [("            if r != request:\n                continue\n", "            if r != request or k > 0:\n                continue\n")], EVICT_PINS),
    ("slid-out page still listed", "alloc", [("                self.pool.free(k, lst[p])\n                lst[p] = -1\n", "                self.pool.free(k, lst[p])\n")], EVICT_PINS),
    ("padding of a table row is page 0", "alloc", [("return lst + [-1] * (width - len(lst))", "return lst + [0] * (width - len(lst))")], EVICT_PINS),
    ("step 1 of five looks at other requests", "alloc", [("mine = self._larges_with_empty(k, self.large_req == request)", "mine = self._larges_with_empty(k, self.large_req != request)")], EVICT_PINS),
    ("an evictable page counts as empty", "alloc", [("return (self.refcount[k] == 0) & ~self.cached[k]", "return (self.refcount[k] == 0)")], EVICT_PINS),
    ("a hit leaves the page evictable", "alloc", [("        self.cached[k][sid] = False\n        self.refcount[k][sid] = 1\n", "        self.refcount[k][sid] = 1\n")], EVICT_PINS),
    ("evicted small page stays cached", "alloc", [("            sid = min(keys)[2]\n            self.cached[k][sid] = False\n", "            sid = min(keys)[2]\n")], EVICT_PINS),
    ("step 5 takes pages of any state", "alloc", [("cand = np.flatnonzero(self.cached[k] & (self.refcount[k] == 0))", "cand = np.flatnonzero(self.refcount[k] >= 0)")], EVICT_PINS),
    ("evicted large page's small pages stay cached", "alloc", [("                self.cached[ko][s] = False           # \"all small pages ... are marked empty\"\n", "                pass\n")], EVICT_PINS),
    ("large pages of equal age: shortest prefix first", "alloc", [("-int(self.prefix_length[ko][ids].max()), large)", "int(self.prefix_length[ko][ids].max()), large)")], EVICT_PINS),
    # ---- Sec. 5.2 / 5.3: hit rules
    ("full-attention prefixes skip a miss", "alloc", [("        if not is_hit[p - 1]:\n            break\n        out.append(p)", "        if not is_hit[p - 1]:\n            continue\n        out.append(p)")], EVICT_PINS),
    ("window rule one token short", "alloc", [("for x in range(window) if p - x >= 1", "for x in range(window - 1) if p - x >= 1")], EVICT_PINS),
    ("window rule shifted by one token", "alloc", [("if all(is_hit[p - x - 1] for x in range(window) if p - x >= 1):", "if all(is_hit[p - x - 2] for x in range(window) if p - x >= 2):")], EVICT_PINS),
    ("state every stride tokens, from zero", "alloc", [("for p in range(stride, len(is_hit) + 1, stride)", "for p in range(1, len(is_hit) + 1, stride)")], EVICT_PINS),
    ("shortest common prefix", "alloc", [("return max(common) if common else 0", "return min(common) if common else 0")], EVICT_PINS),
    ("union instead of intersection", "alloc", [("common &= set(v)", "common |= set(v)")], EVICT_PINS),
    # ---- attention (the textbook definition)
    ("window one token short (attention)", "attn", [("return max(0, seq_len - window), seq_len", "return max(0, seq_len - window + 1), seq_len")], ATTN_PINS),
    ("window excludes the new token", "attn", [("return max(0, seq_len - window), seq_len", "return max(0, seq_len - window - 1), seq_len - 1")], ATTN_PINS),
    ("full attention misses the new token", "attn", [("    return 0, seq_len\n", "    return 0, seq_len - 1\n")], ATTN_PINS),
    ("heads interleaved instead of grouped", "attn", [("kv = h // G", "kv = h % Hkv")], ATTN_PINS),
    ("scale dropped", "attn", [("s = scale * (K[kv, lo:hi, :] @ q[h, :])", "s = (K[kv, lo:hi, :] @ q[h, :])")], ATTN_PINS),
    ("sign of the exponent", "attn", [("e = np.exp(s - m)", "e = np.exp(m - s)")], ATTN_PINS),
    ("no normalisation", "attn", [("out[h, :] = (e @ V[kv, lo:hi, :]) / e.sum()", "out[h, :] = (e @ V[kv, lo:hi, :])")], ATTN_PINS),
    ("values of the whole history", "attn", [("out[h, :] = (e @ V[kv, lo:hi, :]) / e.sum()", "out[h, :] = (e @ V[kv, hi - e.size:hi, :][::-1]) / e.sum()")], ATTN_PINS),
    ("keys used as values", "attn", [("out[h, :] = (e @ V[kv, lo:hi, :]) / e.sum()", "out[h, :] = (e @ K[kv, lo:hi, :]) / e.sum()")], ATTN_PINS),
    ("query of the wrong head", "attn", [("s = scale * (K[kv, lo:hi, :] @ q[h, :])", "s = scale * (K[kv, lo:hi, :] @ q[kv * G, :])")], ATTN_PINS),
]


def _load(name, path, replacements=()):
    src = open(path).read()
    for text, repl in replacements:
        assert src.count(text) == 1, f"{os.path.basename(path)}: {src.count(text)} matches of {text!r}"
        src = src.replace(text, repl)
    mod = types.ModuleType(name)
    mod.__file__ = path
    mod.__package__ = name.rpartition(".")[0]
    exec(compile(src, path, "exec"), mod.__dict__)
    return mod


def _cases(fn):
    """Argument tuples of a pin: the cross product of its parametrize marks; None if it needs fixtures."""
    names, values = [], []
    for mark in getattr(fn, "pytestmark", []):
        if mark.name == "parametrize":
            ns = [n.strip() for n in mark.args[0].split(",")]
            names.append(ns)
            values.append([v.values if hasattr(v, "values") else (v if len(ns) > 1 else (v,)) for v in mark.args[1]])
    flat = [n for ns in names for n in ns]
    if set(inspect.signature(fn).parameters) != set(flat):
        return None
    out = []
    for combo in itertools.product(*values):
        kw = {}
        for ns, vs in zip(names, combo):
            kw.update(dict(zip(ns, vs)))
        out.append(kw)
    return out


def first_failing_pin(which, replacements, pin_files):
    """Runs the pins against the oracle module `which` with `replacements` applied to its source.
    Returns the name of the first pin that fails, or None when all pass."""
    import oracle
    real = sys.modules.get(f"oracle.{which}")
    mutant = _load(f"oracle.{which}", os.path.join(ROOT, "oracle", f"{which}.py"), replacements)
    saved_helpers = sys.modules.pop("helpers", None)
    sys.modules[f"oracle.{which}"] = mutant
    setattr(oracle, which, mutant)
    try:
        for i, fname in enumerate(pin_files):
            pins = _load(f"_pins_{which}_{i}", os.path.join(HERE, fname))
            for name, fn in list(vars(pins).items()):
                if not name.startswith("test_") or not callable(fn):
                    continue
                cases = _cases(fn)
                if cases is None:
                    continue
                for kw in cases:
                    try:
                        fn(**kw)
                    except BaseException as e:      # a pin failed (assertion, or the mistake made it crash)
                        if isinstance(e, (KeyboardInterrupt, SystemExit)):
                            raise
                        return f"{fname}::{name}{kw if kw else ''}: {type(e).__name__}"
        return None
    finally:
        if real is not None:
            sys.modules[f"oracle.{which}"] = real
            setattr(oracle, which, real)
        sys.modules.pop("helpers", None)
        if saved_helpers is not None:
            sys.modules["helpers"] = saved_helpers


@pytest.mark.parametrize("which,pin_files", [("alloc", ALLOC_PINS), ("attn", ATTN_PINS)])
def test_the_unaltered_oracle_passes_its_pins_run_this_way(which, pin_files):
    assert first_failing_pin(which, [], pin_files) is None


@pytest.mark.parametrize("name,which,replacements,pin_files", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(name, which, replacements, pin_files):
    killer = first_failing_pin(which, replacements, pin_files)
    print(f"[mutant] {name}: caught by {killer}")
    assert killer is not None, f"no pin notices: {name}"
