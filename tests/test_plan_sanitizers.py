"""The host-side planning of the library (csrc/fc_plan.cpp: validation, prefix
sums of block counts, request descriptors, work lists; host code, no GPU) under
AddressSanitizer and UndefinedBehaviorSanitizer: the shapes of the five
benchmark configurations plus seeded random valid and invalid arguments must
run clean, give the same plans as an unsanitized build, and agree with the
oracle's bookkeeping (status, block counts, offsets, free blocks afterwards)."""

import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(HERE, "plan_sanitizer_driver.cpp"),
       os.path.join(ROOT, "paper_2503_08461_amd", "csrc", "fc_plan.cpp")]
CODES = {None: 0, "EINVAL": -1, "ENOMEM": -2}
N_LISTS, LIST_ALL, LIST_KNORM, LIST_SNAP, LIST_FUSED = 12, 11, 10, 5, 0


def _build(tmp_path, name, flags):
    exe = str(tmp_path / name)
    subprocess.run(["g++", "-std=c++17", "-O1", "-g"] + flags + SRC + ["-o", exe], check=True)
    return exe


def _run(exe, text):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], input=text, capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    return r.stdout


def _ints(a):
    return " ".join(str(int(x)) for x in a)


class Case:
    """One fc_compress_batch-shaped call."""

    def __init__(self, lens, methods, budgets, n_layers=2, n_heads=3, d=128, n_free=None,
                 mode=0, in_place=False,
                 max_blocks=None, window=32, pool_kernel=7, windows=None, pks=None,
                 need_lse=False, q_ok=True, lse_ok=True, null_mask=0):
        self.lens = np.array(lens, np.int64)
        self.methods = np.array(methods, np.int64)
        self.budgets = np.array(budgets, np.int64)
        self.n_layers, self.n_heads, self.d = n_layers, n_heads, d
        self.mode, self.in_place = mode, in_place
        self.window, self.pool_kernel, self.windows, self.pks = window, pool_kernel, windows, pks
        self.need_lse, self.q_ok, self.lse_ok, self.null_mask = need_lse, q_ok, lse_ok, null_mask
        nb = [fo.blocks_for(max(int(x), 0), 16) for x in self.lens]
        self.max_blocks = max(nb + [1]) if max_blocks is None else max_blocks
        need = sum(fo.blocks_for(int(b), 16) for b, m in zip(self.budgets, self.methods)
                   if m != 0 and b > 0)
        self.n_free = need + 5 if n_free is None else n_free

    def text(self):
        per = self.windows is not None
        head = [self.n_layers, self.n_heads, self.d, self.n_free, self.mode, int(self.in_place),
                len(self.lens), self.max_blocks, int(per),
                self.window, self.pool_kernel, int(self.need_lse), int(self.q_ok),
                int(self.lse_ok), self.null_mask]
        rows = [_ints(self.lens), _ints(self.methods), _ints(self.budgets)]
        if per:
            rows += [_ints(self.windows), _ints(self.pks)]
        return "compress " + _ints(head) + "\n" + "\n".join(rows) + "\n"

    def oracle_status_and_top(self):
        """The oracle's verdict on the same call and, if it accepts, the free
        blocks left after its allocation and reclaim steps (a pool with zero
        layers: bookkeeping only)."""
        n_req = len(self.lens)
        n_old = [fo.blocks_for(max(int(x), 0), 16) for x in self.lens]
        st = fo.FreeStack(self.n_free + sum(n_old))
        bt = np.full((n_req, self.max_blocks + max(n_old + [0])), -1, np.int32)
        for r in range(n_req):
            bt[r, :n_old[r]] = st.alloc(n_old[r])
        bt = bt[:, :max(self.max_blocks, 1)] if self.max_blocks >= max(n_old + [0]) else \
            np.zeros((n_req, max(self.max_blocks, 0)), np.int32)
        lens = self.lens.astype(np.int32).copy()
        window = np.array(self.windows) if self.windows is not None else self.window
        pks = np.array(self.pks) if self.pks is not None else self.pool_kernel
        status = fo.validate_batch(st, bt, lens, window, self.methods, self.budgets, pks, 16,
                                   self.in_place)
        if status is not None:
            return status, None
        skeleton = np.zeros((0, st.n_blocks if hasattr(st, "n_blocks") else len(st.stack), 2,
                             self.n_heads, 16, self.d), np.float16)
        status, _, _ = fo.compress_batch(skeleton, st, bt, lens, None, window, self.methods,
                                         self.budgets, pks, in_place=self.in_place)
        assert status is None
        return None, st.top


def _parse(out):
    """[(kind-specific header ints, {tag: [rows]})] per case."""
    cases = []
    for line in out.splitlines():
        parts = line.split()
        if parts[0] == "R":
            cases.append(([int(x) for x in parts[1:]], {}))
        else:
            cases[-1][1].setdefault(parts[0], []).append([int(x) for x in parts[1:]])
    return cases


def _check_compress(case, header, rows):
    rc, code, total_new, total_old, total_rel, top_after, kept_e, score_e, raw_f, window_hi, \
        n_descs = header
    if len(case.lens) == 0:
        assert rc == 0 and n_descs == 0          # an empty batch is accepted as it is
        return
    status, top = case.oracle_status_and_top()
    assert rc == code == CODES[status], (case.text(), rc, status)
    if status is not None:
        return
    n_lh = case.n_layers * case.n_heads
    comp = [r for r in range(len(case.lens)) if case.methods[r] != 0]
    assert n_descs == len(comp) and top_after == top
    if not comp:
        return
    descs = rows["D"]
    L = case.lens[comp]
    B = case.budgets[comp]
    n_old = np.array([fo.blocks_for(int(x), 16) for x in L])
    n_new = np.array([fo.blocks_for(int(x), 16) for x in B])
    ex = lambda a: np.concatenate([[0], np.cumsum(a)[:-1]])
    if case.windows is None:
        q_off = np.array(comp) * n_lh * case.window * case.d
    else:
        w_all = np.where(case.methods == 1, np.maximum(np.array(case.windows), 0), 0)
        q_off = (np.concatenate([[0], np.cumsum(w_all)[:-1]]) * n_lh * case.d)[comp]
    assert total_old == n_old.sum() and total_rel == (n_old - n_new).sum()
    assert total_new == (0 if case.in_place else n_new.sum())
    assert kept_e == n_lh * B.sum() and score_e == n_lh * L.sum()
    new_off = ex(n_old - n_new) if case.in_place else ex(n_new)
    raw_total = 0
    for i, d in enumerate(descs):
        (row, sl, bud, m, no, nn, old_off, noff, score_off, raw_off, kept_off, qo, win, pk) = d[:14]
        assert (row, sl, bud, m) == (comp[i], L[i], B[i], case.methods[comp[i]])
        assert (no, nn, old_off, noff) == (n_old[i], n_new[i], ex(n_old)[i], new_off[i])
        assert score_off == n_lh * ex(L)[i] and kept_off == n_lh * ex(B)[i] and qo == q_off[i]
        if m == 1:
            assert win == (case.windows[comp[i]] if case.windows is not None else case.window)
    # work lists: every request in exactly one scoring list; heaviest first
    lists = {r[0]: (r[1], r[3:]) for r in rows["L"]}
    assert len(lists) == N_LISTS
    seen = []
    for li, (max_len, idx) in lists.items():
        if li in (LIST_ALL,):
            continue
        seen += idx
        if idx:
            w = [int(L[i]) * (0 if descs[i][3] == 3 else 1 if (descs[i][3] == 2 or case.need_lse)
                              else 2) + 4 * int(B[i]) for i in idx]
            assert w == sorted(w, reverse=True)
        scored = [int(L[i]) for i in idx if descs[i][3] != 3]
        assert max_len == (max(scored) if scored else 0)
    assert sorted(seen) == list(range(len(comp)))
    for li in range(LIST_FUSED, LIST_FUSED + 5):
        for i in lists[li][1]:
            assert descs[i][3] == 3 or (case.mode == 0 and L[i] <= 8192)
            if descs[i][3] == 1:
                assert (descs[i][12] + 15) // 16 == li - LIST_FUSED
    sep = lists[LIST_ALL][1]
    assert sorted(sep) == sorted(lists[LIST_KNORM][1] + sum((lists[LIST_SNAP + c][1] for c in range(5)), []))
    for i in sep:
        raw_total += n_lh * int(L[i])
    assert raw_f == raw_total
    raw_offs = sorted(descs[i][9] for i in sep)
    assert len(set(raw_offs)) == len(raw_offs)


def _config_cases():
    cases = []
    for c in (1, 2, 3, 4, 5):
        wl = synth.make_workload(c)
        for mode in (0, 1):
            cases.append(Case(wl.seq_lens, wl.methods, wl.budgets, wl.n_layers, wl.n_heads,
                              wl.head_dim, mode=mode, window=wl.window,
                              pool_kernel=wl.pool_kernel))
        cases.append(Case(wl.seq_lens, wl.methods, wl.budgets, wl.n_layers, wl.n_heads,
                          wl.head_dim, in_place=True, n_free=0, window=wl.window))
        cases.append(Case(wl.seq_lens, wl.methods, wl.budgets, wl.n_layers, wl.n_heads,
                          wl.head_dim, n_free=3, window=wl.window))          # ENOMEM (or just fits)
    return cases


def _random_cases(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    cases = []
    for _ in range(n):
        R = int(rng.integers(0, 12))
        W = int(rng.integers(1, 65))
        lens, methods, budgets = [], [], []
        for _r in range(R):
            m = int(rng.choice([0, 1, 2, 3]))
            L = int(rng.integers(1, 20000))
            B = int(rng.integers(1, L + 1))
            kind = rng.random()
            if kind < 0.08:
                B = int(rng.choice([0, -3, L + 1]))             # bad budget
            elif kind < 0.12:
                m = int(rng.choice([4, -1, 99]))                # unknown method
            elif kind < 0.16:
                L = int(rng.choice([0, -5]))                    # bad length
                B = 1
            elif m == 1 and kind > 0.25:
                L = max(L, W)
                B = int(rng.integers(W, L + 1))
            lens.append(L); methods.append(m); budgets.append(B)
        kw = dict(n_layers=int(rng.integers(1, 4)), n_heads=int(rng.integers(1, 5)),
                  d=int(rng.choice([64, 128])), mode=int(rng.integers(0, 2)),
                  in_place=bool(rng.integers(0, 2)), window=W,
                  pool_kernel=int(rng.choice([1, 3, 7, 15, 63, 2, 0])))
        if rng.random() < 0.2:
            kw["n_free"] = int(rng.integers(0, 50))             # often too few
        if rng.random() < 0.15:
            kw["max_blocks"] = int(rng.integers(0, 40))         # often too small
        if rng.random() < 0.3:
            kw["windows"] = [int(rng.integers(1, 65)) for _r in range(R)]
            kw["pks"] = [int(rng.choice([1, 3, 5, 63])) for _r in range(R)]
        cases.append(Case(lens, methods, budgets, **kw))
    return cases


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_planning_is_clean_under_asan_and_ubsan_and_agrees_with_the_oracle(tmp_path):
    plain = _build(tmp_path, "plain", [])
    checked = _build(tmp_path, "checked",
                     ["-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                      "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan"])
    cases = _config_cases() + _random_cases(400, 2024)
    text = "".join(c.text() for c in cases)
    out = _run(checked, text)
    assert out == _run(plain, text)
    parsed = _parse(out)
    assert len(parsed) == len(cases)
    accepted = 0
    for case, (header, rows) in zip(cases, parsed):
        _check_compress(case, header, rows)
        accepted += header[0] == 0
    assert 100 < accepted < len(cases) - 50          # both outcomes are well represented

    # refusals that come from the library's own limits and argument checks
    ok = dict(lens=[5000, 300], methods=[1, 2], budgets=[900, 100], window=32)
    bad = [Case(**ok, null_mask=1), Case(**ok, null_mask=2), Case(**ok, null_mask=4),
           Case(**ok, q_ok=False), Case(**ok, need_lse=True, lse_ok=False),
           Case(lens=[5000], methods=[1], budgets=[900], window=65),
           Case(lens=[5000], methods=[1], budgets=[900], window=32, pool_kernel=65),
           Case(lens=[32769], methods=[2], budgets=[900]),
           Case(lens=[5000, 300], methods=[1, 1], budgets=[900, 100], windows=[32, 16], pks=[7, 3],
                null_mask=8)]
    for (header, _rows), case in zip(_parse(_run(checked, "".join(c.text() for c in bad))), bad):
        assert header[0] == -1, case.text()
    # the same valid call goes through
    header, rows = _parse(_run(checked, Case(**ok, mode=1).text()))[0]
    assert header[0] == 0 and len(rows["D"]) == 2

    # the other planners: window log-sum-exp, chunk MLP, append, decode attention
    other = ("lse 2 3 128 4 80 32 1\n700 100 1200 64\n1 2 1 1\n"
             "lse 2 3 128 2 80 32 0\n700 20\n"
             "mlp 2 2 64 100 3 80 5 256 1\n640 100 1200\n35 0 1200\n611 100 1200\n1 0 1\n"
             "mlp 2 2 64 1 1 80 5 256 0\n640\n35\n611\n"
             "mlp 2 2 64 100 1 80 5 256 0\n640\n50\n40\n"
             "append 1 1 64 1 4 8 0\n15 16 0 33\n"
             "append 1 1 64 9 4 8 1\n15 16 127 128\n1 1 1 1\n"
             "decode 2 2 64 3 8 1\n100 50 7\n10 50 0\n"
             "decode 2 2 64 2 8 1\n100 50\n101 50\n")
    out = _run(checked, other)
    assert out == _run(plain, other)
    p = _parse(out)
    assert p[0][0] == [0, 3] and [d[1] for d in p[0][1]["D"]] == [1200, 700, 64]   # longest first
    assert [d[11] for d in p[0][1]["D"]] == [2 * 6 * 32 * 128, 0, 3 * 6 * 32 * 128]  # q offsets by row
    assert p[1][0][0] == -1                                                          # 20 < window
    # 640 tokens, image [35, 611), k = 5: 7 + 116 + 6 chunks = 129 rows -> 9 blocks; 1200 all text: 240
    assert p[2][0][:3] == [0, 9 + 15, 40 + 75] and p[2][0][4] == 100 - 24 + 115
    assert [d[16:19] for d in p[2][1]["D"]] == [[7, 116, 6], [240, 0, 0]]
    assert [j[:3] for j in p[2][1]["J"]] == [[0, 0, 13], [0, 1, 116], [1, 0, 240]]
    # tiles of 256 rows over 8 (layer, head, K|V) units: ceil(8*13/256) = 1, ceil(8*116/256) = 4
    assert [j[3] for j in p[2][1]["J"]] == [0, 1, 1 + 4]
    assert p[3][0][0] == -2 and p[4][0][0] == -1
    assert p[5][0][:2] == [-2, 2]                                  # two requests need a block, one free
    assert p[6][0][0] == -1                                        # table row of 8 entries is full at 128
    assert p[7][0][0] == 0 and p[7][0][2] == 4 * (10 + 50 + 0)
    assert [q[0] for q in p[7][1]["Q"]] == [1, 0, 2]               # largest budget first
    assert p[8][0][0] == -1
