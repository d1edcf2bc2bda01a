"""Do the pins bite?  (CPU only; every mistake is planted in a COPY of the oracle's source.)

Each case below rewrites one line of `oracle/attention.py` or `oracle/kvfs_model.py` into a
plausible mistake (a dropped scale, a wrong head mapping, an off-by-one mask, K and V swapped, the
page with the highest rank instead of the lowest, a copy-on-write that is skipped, ...), loads the
rewritten text in place of the module, re-runs the pin files against it, and requires that at
least one pin fails.  The unmodified text must pass every pin under the same harness.
(Rewrites that change nothing observable are not listed: e.g. a removed file whose name stays
behaves exactly like the new empty file that the next open of the name creates.)"""
import importlib.util
import inspect
import os
import sys

import pytest

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_TESTS = os.path.join(_ROOT, "tests")


def _load(name, path, text=None):
    spec = importlib.util.spec_from_file_location(name, path)
    mod = importlib.util.module_from_spec(spec)
    sys.modules[name] = mod
    if text is None:
        spec.loader.exec_module(mod)
    else:
        exec(compile(text, path, "exec"), mod.__dict__)
    return mod


def _cases(fn):
    """The calls pytest would make: one per parametrize row, or one without arguments."""
    marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
    params = list(inspect.signature(fn).parameters)
    if not marks:
        return [()] if not params else []            # a test that takes fixtures is left out
    names = [s.strip() for s in marks[0].args[0].split(",")]
    if len(marks) != 1 or params != names:
        return []
    return [tuple(v) if len(names) > 1 else (v,) for v in marks[0].args[1]]


def _failing_pins(module_file, edits, pin_files, only=None, first=False, skip=()):
    """Pins (function names) that fail when `module_file` of the oracle carries `edits`.
    only: run just these functions; skip: not these (a caller that lives in a pin file names itself);
    first: stop at the first one that fails."""
    path = os.path.join(_ROOT, "oracle", module_file)
    text = open(path).read()
    for old, new in edits:
        assert text.count(old) == 1, f"mutation point not unique or gone: {old!r}"
        text = text.replace(old, new)
    touched = ["oracle.attention", "oracle.kvfs_model", "oracle.driver", "oracle.scheduler", "oracle"]
    saved = {k: sys.modules.get(k) for k in touched}
    import oracle                                   # the package itself stays; its submodules are swapped
    saved_attrs = {k: getattr(oracle, k, None) for k in ("attention", "kvfs_model", "driver", "scheduler")}
    failed = []
    try:
        # dependency order: the state model, attention, then the driver that imports both
        for name, file in (("oracle.kvfs_model", "kvfs_model.py"), ("oracle.attention", "attention.py"), ("oracle.driver", "driver.py"),
                           ("oracle.scheduler", "scheduler.py")):
            _load(name, os.path.join(_ROOT, "oracle", file), text if file == module_file else None)
        for pf in pin_files:
            pins = _load("pins_under_mutation_" + pf[:-3], os.path.join(_TESTS, pf))
            for name, fn in sorted(vars(pins).items()):
                if not name.startswith("test_") or not callable(fn) or (only is not None and name not in only) or name in skip:
                    continue
                if first and failed:
                    break
                for args in _cases(fn):
                    try:
                        fn(*args)
                    except (Exception, pytest.fail.Exception):   # a wrong result, a missing error or a crash: the mistake did not pass
                        failed.append(name)
                        break
            del sys.modules["pins_under_mutation_" + pf[:-3]]
    finally:
        for k, v in saved.items():
            if v is None:
                sys.modules.pop(k, None)
            else:
                sys.modules[k] = v
        for k, v in saved_attrs.items():
            if v is not None:
                setattr(oracle, k, v)
    return failed


_SCHED_PINS = ["test_oracle_scheduler.py"]
_ATTN_PINS = ["test_oracle_attention.py"]
_KVFS_PINS = ["test_oracle_kvfs.py", "test_oracle_attention.py"]


def test_unmodified_oracle_passes_under_the_harness():
    assert _failing_pins("attention.py", [], _ATTN_PINS) == []
    assert _failing_pins("kvfs_model.py", [], _KVFS_PINS) == []
    assert _failing_pins("scheduler.py", [], _SCHED_PINS) == []
    assert _failing_pins("driver.py", [], _ATTN_PINS) == []


@pytest.mark.parametrize("what,edits", [
    ("scale dropped", [("@ K[:, g, :].T) * scale", "@ K[:, g, :].T)")]),
    ("scale 1/D", [("1.0 / np.sqrt(D)", "1.0 / D")]),
    ("sign of the scores", [("@ K[:, g, :].T) * scale", "@ K[:, g, :].T) * -scale")]),
    ("heads interleaved instead of grouped", [("g = h // G", "g = h % Hkv")]),
    ("a token does not see itself", [("<= (len_before + np.arange(n))", "< (len_before + np.arange(n))")]),
    ("a token sees one token too many", [("<= (len_before + np.arange(n))", "<= (len_before + 1 + np.arange(n))")]),
    ("no causal mask", [("s = np.where(visible, s, dtype(-np.inf))", "pass")]),
    ("weights not normalised", [("p = e / e.sum(axis=1, keepdims=True)", "p = e")]),
    ("normalised over the rows", [("p = e / e.sum(axis=1, keepdims=True)", "p = e / e.sum(axis=0, keepdims=True)")]),
    ("weighted sum of K", [("out[:, h, :] = p @ V[:, g, :]", "out[:, h, :] = p @ K[:, g, :]")]),
    ("K and V swapped in the gather", [("K[lo:lo + n] = pg[0,", "K[lo:lo + n] = pg[1,"), ("V[lo:lo + n] = pg[1,", "V[lo:lo + n] = pg[0,")]),
    ("every page read from slot 0 of the table", [("pg = pool.page(p)", "pg = pool.page(page_ids[0])")]),
    ("rows of the batch not advanced", [("        t += n\n    return out", "        t += 0\n    return out")]),
    ("file length before the append passed as 0", [("dense_attention(q[t:t + n], K, V, L, dtype=dtype)", "dense_attention(q[t:t + n], K[:n], V[:n], 0, dtype=dtype)")]),
])
@pytest.mark.filterwarnings("ignore::RuntimeWarning")       # a rewritten mask can leave a row with no visible token
def test_a_mistake_in_the_attention_oracle_fails_a_pin(what, edits):
    failed = _failing_pins("attention.py", edits, _ATTN_PINS)
    print(f"[{what}] caught by: {', '.join(failed)}")
    assert failed, f"no pin notices: {what}"


@pytest.mark.parametrize("what,edits", [
    ("highest rank first", [("heapq.heappop(self.free_ranks)", "self.free_ranks.pop(self.free_ranks.index(max(self.free_ranks)))")]),
    ("fork does not count references", [("            self.refcount[p] += 1\n", "            self.refcount[p] += 0\n")]),
    ("shared partial page written in place", [("if r != 0 and self.refcount[f.pages[-1]] > 1:", "if False:")]),
    ("partial page always copied", [("if r != 0 and self.refcount[f.pages[-1]] > 1:", "if r != 0:")]),
    ("copy leaves the source's count alone", [("                self.refcount[src] -= 1\n", "                pass\n")]),
    ("copy takes one slot too few", [("cow.append((src, dst, r))", "cow.append((src, dst, r - 1))")]),
    ("full page copied too", [("if r != 0 and self.refcount[f.pages[-1]] > 1:", "if len(f.pages) > 0 and self.refcount[f.pages[-1]] > 1:")]),
    ("new page one token late", [("                if f.length % self.P == 0:\n", "                if f.length % self.P == 1:\n")]),
    ("freed page never returns", [("        if self.refcount[p] == 0:\n", "        if self.refcount[p] < 0:\n")]),
    ("copies after the appends", [("        for src, dst, r in cow:\n            self.copy_slots(src, dst, r)\n        t = 0\n", "        t = 0\n"),
                                  ("        assert t == len(k_new)\n", "        assert t == len(k_new)\n        for src, dst, r in cow:\n            self.copy_slots(src, dst, r)\n")]),
    ("K written into the V half", [("        pg[0, :, slot, :] = k_row\n        pg[1, :, slot, :] = v_row\n", "        pg[1, :, slot, :] = k_row\n        pg[0, :, slot, :] = v_row\n")]),
    ("second open of a name makes a new file", [("if name is not None and name in self.names:", "if False:")]),
    ("close of the last handle keeps an anonymous file", [("if f.name is None and not f.handles:", "if False:")]),
    ("truncate keeps one page too few", [("keep=-(-new_len // self.P))", "keep=new_len // self.P)")]),
    ("truncate keeps every page", [("keep=-(-new_len // self.P))", "keep=len(f.pages))")]),
    ("truncate past the end allowed", [("if new_len < 0 or new_len > f.length:", "if new_len < 0:")]),
    ("extract: a page in any slot order is shared", [("same = all(pg == toks[0][0] and sl == k for k, (pg, sl) in enumerate(toks))", "same = all(pg == toks[0][0] for pg, sl in toks)")]),
    ("extract: nothing is ever shared", [("same = all(pg == toks[0][0] and sl == k for k, (pg, sl) in enumerate(toks))", "same = False")]),
    ("extract: shared page not counted", [("            if s is not None:\n                self.refcount[s] += 1\n", "            if s is not None:\n")]),
    ("extract: destination slots shifted", [("moves.append((pg, sl, dst, k))", "moves.append((pg, sl, dst, (k + 1) % P))")]),
    ("extract of no tokens skips the check of its source", [("        self._file(h, usable=True)                        # the source must exist and not wait, even for no tokens\n", "")]),
    ("extract: index past the end allowed", [("if i < 0 or i >= f.length:", "if i < 0 or i > f.length:")]),
    ("merge: second file first", [("for h in handles for i in range(", "for h in reversed(handles) for i in range(")]),
    ("offload: a page leaves as soon as one reader waits", [("if len(self.waiters[p]) == self.refcount[p]:", "if True:")]),
    ("offload: host slots never reused", [("                    if self.free_slots:\n", "                    if False:\n")]),
    ("offload: the page is not freed", [("                    self.refcount[p] = 0\n                    heapq.heappush(self.free_ranks, int(self.rank[p]))\n", "")]),
    ("restore: only the restored file's entry is rewritten", [("                for g, j in refs:\n                    g.pages[j] = q\n                self.refcount[q] = len(refs)", "                f.pages[i] = q\n                self.refcount[q] = len(refs)")]),
    ("restore: count of the new page is 1", [("self.refcount[q] = len(refs)", "self.refcount[q] = 1")]),
    ("restore: no room check", [("        if len(need) > len(self.free_ranks):\n            raise KVError(ENOSPC, \"page pool exhausted\")\n        out = []\n        for f in files:\n            f.waiting = False", "        out = []\n        for f in files:\n            f.waiting = False")]),
    ("a waiting file can be appended to", [("        if usable and f.waiting:", "        if False:")]),
    ("same file twice in a batch allowed", [("            if any(f is g for g in files):\n                raise KVError(EBUSY, \"same file twice in a batch\")\n", "")]),
    ("batch that does not fit is started anyway", [("        if self.pages_needed(items) > len(self.free_ranks):\n            raise KVError(ENOSPC, \"page pool exhausted\")\n        cow, slots = [], []", "        cow, slots = [], []")]),
])
def test_a_mistake_in_the_state_model_fails_a_pin(what, edits):
    failed = _failing_pins("kvfs_model.py", edits, _KVFS_PINS)
    print(f"[{what}] caught by: {', '.join(failed)}")
    assert failed, f"no pin notices: {what}"


@pytest.mark.parametrize("what,edits", [
    ("rate is the mean gap, not its inverse", [("return 1.0 / self.mean_gap if", "return self.mean_gap if")]),
    ("new gaps ignored", [("self.mean_gap = self.mean_gap + self.w * (gap - self.mean_gap)", "pass")]),
    ("slope with the wrong sign", [("c = (self.mbs - self.mb * self.ms) / var", "c = (self.mb * self.ms - self.mbs) / var")]),
    ("intercept without the slope", [("a = self.ms - self.c * self.mb", "a = self.ms")]),
    ("target ignores the per-call cost", [("t = lam * self.a / (1.0 - load)", "t = lam * self.a")]),
    ("target divided by the load", [("t = lam * self.a / (1.0 - load)", "t = lam * self.a / load if load > 0 else 1.0")]),
    ("overload waits for one call", [("        if load >= 1.0:\n            return float(self.max_batch)", "        if load >= 1.0:\n            return 1.0")]),
    ("never waits", [("        if missing / lam > left:\n            return q                                    # the target is out of reach before the deadline\n        return 0", "        return q")]),
    ("waits although the target is out of reach", [("        if missing / lam > left:\n            return q                                    # the target is out of reach before the deadline\n", "")]),
    ("fires more than max_batch", [("q = min(len(self.pending), self.max_batch)", "q = len(self.pending)")]),
    ("fires while the GPU is busy", [("if not gpu_idle or not self.pending:", "if not self.pending:")]),
])
def test_a_mistake_in_the_scheduler_oracle_fails_a_pin(what, edits):
    failed = _failing_pins("scheduler.py", edits, _SCHED_PINS)
    print(f"[{what}] caught by: {', '.join(failed)}")
    assert failed, f"no pin notices: {what}"


@pytest.mark.parametrize("what,edits", [
    ("bf16 patterns widened into the wrong bits", [("<< np.uint32(16)", "<< np.uint32(15)")]),
    ("sampled rows start at the LIP's index", [("            out[starts[b]:starts[b] + n] = dense_attention(q[starts[b]:starts[b] + n]", "            out[b:b + n] = dense_attention(q[b:b + n]")]),
    ("sampled LIPs read the first LIP's file", [("K, V = gather_file(self.pool, self.model.kv_pages(h), before[b] + n)", "K, V = gather_file(self.pool, self.model.kv_pages(items[0][0]), before[b] + n)")]),
    ("a fork is a fork of the newest file", [("self.h[op[1]] = self.model.kv_fork(self.h[op[2]])", "self.h[op[1]] = self.model.kv_fork(self.h[max(self.h)])")]),
    ("extract moves are not carried out", [("                self.h[op[1]], moves = self.model.kv_extract(self.h[op[2]], op[3])\n                self.pool.move_tokens(moves)\n", "                self.h[op[1]], moves = self.model.kv_extract(self.h[op[2]], op[3])\n")]),
])
@pytest.mark.filterwarnings("ignore::RuntimeWarning")
def test_a_mistake_in_the_oracle_driver_fails_a_pin(what, edits):
    failed = _failing_pins("driver.py", edits, _ATTN_PINS)
    print(f"[{what}] caught by: {', '.join(failed)}")
    assert failed, f"no pin notices: {what}"
