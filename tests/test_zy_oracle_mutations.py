"""Every rule of the oracle listed here is held by a pin: each entry below plants one mistake (a dropped term, a flipped
comparison, a swapped tie rule) in a temporary copy of the oracle's C source, on the CPU, and the named pin file
must fail against that copy.  The oracle under oracle/ is never touched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (what is planted, the pin file that notices it (None: some file of tests/test_oracle_*.py), text in
# oracle/ccld_oracle.c, its replacement)
MUTATIONS = [
    ('mad leg enter removed', 'test_oracle_chains.py',
     '(__int128)le * (__int128)P[P_KMAD_DEN] > (__int128)P[P_KMAD_NUM] * (__int128)S[SEG_ENTER_MAD])',
     '1)'),
    ('mad leg exit removed', 'test_oracle_pins.py',
     '(__int128)lx * (__int128)P[P_KMAD_DEN] > (__int128)P[P_KMAD_NUM] * (__int128)S[SEG_EXIT_MAD])',
     '1)'),
    ('kmad swapped enter', 'test_oracle_chains.py',
     '(__int128)le * (__int128)P[P_KMAD_DEN] > (__int128)P[P_KMAD_NUM] *',
     '(__int128)le * (__int128)P[P_KMAD_NUM] > (__int128)P[P_KMAD_DEN] *'),
    ('kmad swapped exit', 'test_oracle_pins.py',
     '(__int128)lx * (__int128)P[P_KMAD_DEN] > (__int128)P[P_KMAD_NUM] *',
     '(__int128)lx * (__int128)P[P_KMAD_NUM] > (__int128)P[P_KMAD_DEN] *'),
    ('mad leg >= enter', 'test_oracle_pins.py',
     '(__int128)le * (__int128)P[P_KMAD_DEN] > (__int128)P[P_KMAD_NUM]',
     '(__int128)le * (__int128)P[P_KMAD_DEN] >= (__int128)P[P_KMAD_NUM]'),
    ('floor >= enter', 'test_oracle_pins.py',
     'if (le > P[P_LAG_FLOOR_NS] &&',
     'if (le >= P[P_LAG_FLOOR_NS] &&'),
    ('floor >= exit', 'test_oracle_pins.py',
     'if (lx > P[P_LAG_FLOOR_NS] &&',
     'if (lx >= P[P_LAG_FLOOR_NS] &&'),
    ('blame lag direction', 'test_oracle_pins.py',
     'if (sa != sb) return sa > sb ? -1 : 1;',
     'if (sa != sb) return sa < sb ? -1 : 1;'),
    ('blame rank tie desc', 'test_oracle_pins.py',
     'return a < b ? -1 : (a > b ? 1 : 0);\n}\n\n/* ----',
     'return a > b ? -1 : (a < b ? 1 : 0);\n}\n\n/* ----'),
    ('blame flags direction', 'test_oracle_pins.py',
     'if (na != nb) return na > nb ? -1 : 1;',
     'if (na != nb) return na < nb ? -1 : 1;'),
    ('complete ignores inflight', 'test_oracle_pins.py',
     'int complete = (nn == T->size[c]) && n_infl == 0;',
     'int complete = (nn == T->size[c]);'),
    ('fewest tie larger R', 'test_oracle_hang.py',
     '(a == b && (PQ(q, PAIR_RECV) < PQ(best, PAIR_RECV) ||',
     '(a == b && (PQ(q, PAIR_RECV) > PQ(best, PAIR_RECV) ||'),
    ('fewest tie larger rank', 'test_oracle_hang.py',
     'PQ(q, PAIR_RANK) < PQ(best, PAIR_RANK)))))',
     'PQ(q, PAIR_RANK) > PQ(best, PAIR_RANK)))))'),
    ('backpressure >', 'test_oracle_hang.py',
     'PQ(q, PAIR_SENT) - PQ(succ, PAIR_RECV) >= P[P_FIFO_DEPTH]',
     'PQ(q, PAIR_SENT) - PQ(succ, PAIR_RECV) > P[P_FIFO_DEPTH]'),
    ('starved >', 'test_oracle_frames.py',
     'PQ(q, PAIR_RECV) >= PQ(pred, PAIR_SENT)',
     'PQ(q, PAIR_RECV) > PQ(pred, PAIR_SENT)'),
    ('onset min', 'test_oracle_hang.py',
     'if (on > onset) onset = on;',
     'if (ch == 0 || on < onset) onset = on;'),
    ('stalled ch0 only', 'test_oracle_hang.py',
     'if (can_stall) {\n          const cell_t *o',
     'if (can_stall && ch == 0) {\n          const cell_t *o'),
    ('tree deficit any', 'test_oracle_hang.py',
     'if (def[q] == worst) { is_cand[off + q] = 1; ++n_c; }',
     'if (def[q] > 0) { is_cand[off + q] = 1; ++n_c; }'),
    ('rate tie larger rank', 'test_oracle_rates.py',
     'return rank_a < rank_b;',
     'return rank_a > rank_b;'),
    ('theta >=', 'test_oracle_pins.py',
     '(__int128)(tmax - tbase) * (__int128)P[P_THETA_DEN] > (__int128)P[P_THETA_NUM]',
     '(__int128)(tmax - tbase) * (__int128)P[P_THETA_DEN] >= (__int128)P[P_THETA_NUM]'),
    ('beta >=', 'test_oracle_pins.py',
     'if (num > (__int128)P[P_BETA_NUM] * den) cls = 1;',
     'if (num >= (__int128)P[P_BETA_NUM] * den) cls = 1;'),
    ('alpha <=', 'test_oracle_pins.py',
     'else if (num < (__int128)P[P_ALPHA_NUM] * den) cls = 2;',
     'else if (num <= (__int128)P[P_ALPHA_NUM] * den) cls = 2;'),
    ('eq2 tie last', 'test_oracle_pins.py',
     'if (k == k0 || range > best) { best = range; kstar = k; }',
     'if (k == k0 || range >= best) { best = range; kstar = k; }'),
    ('eq2 max dur', 'test_oracle_pins.py',
     'int64_t range = S[SEG_DUR_MAX] - S[SEG_DUR_MIN];\n      if (k == k0',
     'int64_t range = S[SEG_DUR_MAX];\n      if (k == k0'),
    ('tbase rounds <=', 'test_oracle_pins.py',
     'G->cnt < (uint64_t)P[P_TBASE_ROUNDS] &&',
     'G->cnt <= (uint64_t)P[P_TBASE_ROUNDS] &&'),
    ('warmup <', 'test_oracle_pins.py',
     'S[SEG_ENTER_MIN] - G->t0 <= P[P_TBASE_WARMUP_NS]',
     'S[SEG_ENTER_MIN] - G->t0 < P[P_TBASE_WARMUP_NS]'),
    ('dynamic >=', 'test_oracle_pins.py',
     'int dynamic = G->frozen && items[kstar].seq > G->baseline_last_seq;',
     'int dynamic = G->frozen && items[kstar].seq >= G->baseline_last_seq;'),
    ('repeat >', 'test_oracle_pins.py',
     'O[GRP_LOCATE] = slow && G->repeats >= (uint64_t)P[P_REPEAT_THRESHOLD];',
     'O[GRP_LOCATE] = slow && G->repeats > (uint64_t)P[P_REPEAT_THRESHOLD];'),
    ('barrier <=', 'test_oracle_pins.py',
     '(bytes[i0] < (uint64_t)P[P_BARRIER_BYTES]);',
     '(bytes[i0] <= (uint64_t)P[P_BARRIER_BYTES]);'),
    ('hang thr >=', 'test_oracle_pins.py',
     'if (n_infl > 0 && !barrier && now_ns - infl_enter_min > P[P_HANG_THRESHOLD_NS]) {',
     'if (n_infl > 0 && !barrier && now_ns - infl_enter_min >= P[P_HANG_THRESHOLD_NS]) {'),
    ('root1 argmax', 'test_oracle_pins.py',
     'if (cls != 2) root1 = Sx[SEG_ARGMIN_RANK];',
     'if (cls != 2) root1 = Sx[SEG_ARGMAX_RANK];'),
    ('mean ceil', 'test_oracle_pins.py',
     'G->tbase_dyn = G->sum / (int64_t)G->cnt;',
     'G->tbase_dyn = (G->sum + (int64_t)G->cnt - 1) / (int64_t)G->cnt;'),
    ('baseline uses dmin', 'test_oracle_pins.py',
     'G->sum += S[SEG_DUR_MAX]; G->cnt += 1;',
     'G->sum += S[SEG_DUR_MIN]; G->cnt += 1;'),
    ('victim filter off', 'test_oracle_frames.py',
     'if (T->members[p2] == r && R->pair[p2 * PAIR_NCOL + PAIR_ENTERED]) { drop[p] = 1; break; }',
     'if (0) { drop[p] = 1; break; }'),
    ('victim needs entered', 'test_oracle_hang.py',
     'if (T->members[p2] == r && R->pair[p2 * PAIR_NCOL + PAIR_ENTERED]) { drop[p] = 1; break; }',
     'if (T->members[p2] == r) { drop[p] = 1; break; }'),
    ('hung needs stalled', 'test_oracle_hang.py',
     'const int hung = !idle_ok && any_stalled;',
     'const int hung = !idle_ok;'),
    ('cls log2 ceil', 'test_oracle_pins.py',
     'static int floor_log2_u64(uint64_t b) { int c = 0; if (b == 0) b = 1; while (b >>= 1) ++c; return c; }',
     'static int floor_log2_u64(uint64_t b) { int c = 0; if (b == 0) b = 1; b = 2*b-1; while (b >>= 1) ++c; return c; }'),
    ('lag uses min', 'test_oracle_pins.py',
     'int64_t le = t_enter[i] - S[SEG_ENTER_MED], lx',
     'int64_t le = t_enter[i] - S[SEG_ENTER_MIN], lx'),
    ('stall window off by one', 'test_oracle_hang.py',
     'const cell_t *o = s + (L - (uint32_t)W);',
     'const cell_t *o = s + (L - (uint32_t)W + 1);'),
    ('inconsistent op ignored', 'test_oracle_pins.py',
     'if (op[i] != op[i0] || bytes[i] != bytes[i0]) consistent = 0;',
     'if (bytes[i] != bytes[i0]) consistent = 0;'),
    ('alert age from enter_min', 'test_oracle_pins.py',
     'A[ALR_AGE] = now_ns - S[SEG_INFLIGHT_ENTER_MIN];',
     'A[ALR_AGE] = now_ns - S[SEG_ENTER_MIN];'),
    ('median upper', 'test_oracle_chains.py',
     'return scratch[(n - 1) / 2];',
     'return scratch[n / 2];'),
    ('chain prev exit >= enter allowed', 'test_oracle_chains.py',
     't_exit[i] == ORC_INFLIGHT || t_exit[i] > t_enter[self]) continue;',
     't_exit[i] == ORC_INFLIGHT || t_exit[i] >= t_enter[self]) continue;'),
    ('chain prev smallest exit', 'test_oracle_chains.py',
     'if (t_exit[i] != t_exit[prev]) { if (t_exit[i] > t_exit[prev]) prev = i; continue; }',
     'if (t_exit[i] != t_exit[prev]) { if (t_exit[i] < t_exit[prev]) prev = i; continue; }'),
    ('chain prev tie enter smaller', 'test_oracle_chains.py',
     'if (t_enter[i] != t_enter[prev]) { if (t_enter[i] > t_enter[prev]) prev = i; continue; }',
     'if (t_enter[i] != t_enter[prev]) { if (t_enter[i] < t_enter[prev]) prev = i; continue; }'),
    ('chain prev tie comm smaller', 'test_oracle_chains.py',
     'if (comm[i] != comm[prev]) { if (comm[i] > comm[prev]) prev = i; continue; }',
     'if (comm[i] != comm[prev]) { if (comm[i] < comm[prev]) prev = i; continue; }'),
    ('chain parent smallest lag', 'test_oracle_chains.py',
     'if (best < 0 || Q[FLG_LAG_ENTER] > flag[best * FLG_NCOL + FLG_LAG_ENTER] ||',
     'if (best < 0 || Q[FLG_LAG_ENTER] < flag[best * FLG_NCOL + FLG_LAG_ENTER] ||'),
    ('chain parent tie larger rank', 'test_oracle_chains.py',
     'Q[FLG_RANK] < flag[best * FLG_NCOL + FLG_RANK]))\n        best',
     'Q[FLG_RANK] > flag[best * FLG_NCOL + FLG_RANK]))\n        best'),
    ('chain parent late exit counts', 'test_oracle_chains.py',
     'Q[FLG_SEQ] != (int64_t)seq[prev] || !(Q[FLG_KIND] & FLAG_LATE_ENTER)) continue;',
     'Q[FLG_SEQ] != (int64_t)seq[prev]) continue;'),
    ('chain late exit gets a parent', 'test_oracle_chains.py',
     "if (!(F[FLG_KIND] & FLAG_LATE_ENTER)) continue;\n    /* the flag's own record */",
     "/* the flag's own record */"),
    ('chain caused by own rank', 'test_oracle_chains.py',
     'per_rank[chain[k * CHN_NCOL + CHN_ROOT_RANK] * CHR_NCOL + CHR_CAUSED] += 1;',
     'per_rank[F[FLG_RANK] * CHR_NCOL + CHR_CAUSED] += 1;'),
    ('window: member error before unknown communicator', None,
     '  if (bad_comm) { R->status = ORC_E_UNKNOWN_COMM; return R->status; }\n  if (bad_member) { R->status = ORC_E_RANK_NOT_MEMBER; return R->status; }',
     '  if (bad_member) { R->status = ORC_E_RANK_NOT_MEMBER; return R->status; }\n  if (bad_comm) { R->status = ORC_E_UNKNOWN_COMM; return R->status; }'),
    ('window: range error before member error', None,
     '  if (bad_member) { R->status = ORC_E_RANK_NOT_MEMBER; return R->status; }\n  if (bad_range) { R->status = ORC_E_RANGE; return R->status; }',
     '  if (bad_range) { R->status = ORC_E_RANGE; return R->status; }\n  if (bad_member) { R->status = ORC_E_RANK_NOT_MEMBER; return R->status; }'),
    ('window: exit before enter allowed', None,
     't_enter[i] == ORC_INFLIGHT || t_exit[i] < t_enter[i]) bad_range = 1;',
     't_enter[i] == ORC_INFLIGHT) bad_range = 1;'),
    ('window: op 16 allowed', None,
     'if (op[i] >= OP_MAX || t_enter[i] < 0',
     'if (op[i] > OP_MAX || t_enter[i] < 0'),
    ('window: negative enter allowed', None,
     'if (op[i] >= OP_MAX || t_enter[i] < 0 ||',
     'if (op[i] >= OP_MAX ||'),
    ('snapshots: range before member', None,
     '  if (bad_member) return ORC_E_RANK_NOT_MEMBER;\n  if (bad_range) return ORC_E_RANGE;\n  cell_t *cell',
     '  if (bad_range) return ORC_E_RANGE;\n  if (bad_member) return ORC_E_RANK_NOT_MEMBER;\n  cell_t *cell'),
    ('snapshots: gap before duplicate', None,
     '  if (dup) { free(cell); return ORC_E_DUPLICATE_KEY; }\n  if (gap) { free(cell); return ORC_E_SNAPSHOT_GAP; }',
     '  if (gap) { free(cell); return ORC_E_SNAPSHOT_GAP; }\n  if (dup) { free(cell); return ORC_E_DUPLICATE_KEY; }'),
    ('snapshots: channel == n_ch allowed', None,
     'if (snap[i] >= n_snap || channel[i] >= n_ch) bad_range = 1;',
     'if (snap[i] >= n_snap || channel[i] > n_ch) bad_range = 1;'),
    ('rates: open run counted', None,
     '        while (open > 0 && s[open - 1].seq == s[n_snap - 1].seq) --open;',
     '        open = n_snap;'),
    ('rates: first sample compared with the previous run', None,
     '          uint32_t ps = 0, pr = 0;\n          int64_t cs = 0, cr = 0;',
     '          uint32_t ps = t ? s[t - 1].sent : 0, pr = t ? s[t - 1].recv : 0;\n          int64_t cs = 0, cr = 0;'),
    ('rates: run without change counted as operation', None,
     '          if (cs) { Q[RATE_OPS_SEND] += 1; Q[RATE_CHG_SEND] += cs; }',
     '          { Q[RATE_OPS_SEND] += 1; Q[RATE_CHG_SEND] += cs; }'),
    ('rates: recv changes from sends', None,
     '            if (s[t].recv != pr) ++cr;',
     '            if (s[t].sent != ps) ++cr;'),
    ('rates: root ignores recv', None,
     '        if (H[RC_ROOT] == ORC_NO_RANK || rate_less(Q[RATE_OPS_RECV], Q[RATE_CHG_RECV], rk, bb[0], bb[1], H[RC_ROOT])) {',
     '        if (0) {'),
    ('rates: maximal rate', None,
     '  if (l != r) return l < r;',
     '  if (l != r) return l > r;'),
    ('frames: smaller counter wins', None,
     '        if (cnt2 > cnt || (cnt2 == cnt && b2 > b)) loses = 1;',
     '        if (cnt2 < cnt || (cnt2 == cnt && b2 > b)) loses = 1;'),
    ('frames: equal counters smaller block wins', None,
     '        if (cnt2 > cnt || (cnt2 == cnt && b2 > b)) loses = 1;',
     '        if (cnt2 > cnt || (cnt2 == cnt && b2 < b)) loses = 1;'),
    ('frames: older frame overwrites', None,
     '        if (cnt < L->seq) continue;                 /* what is remembered is newer */',
     ''),
    ('frames: unwritten blocks decoded', None,
     '      if (!(rd_u32(B + 4) & 1u)) continue;\n      const uint32_t c = rd_u32(B);\n      const uint64_t cnt = rd_u64(B + 8);',
     '      const uint32_t c = rd_u32(B);\n      const uint64_t cnt = rd_u64(B + 8);'),
    ('frames: channels beyond the header keep counts', None,
     '        L->sent = ch < nch ? (uint32_t)rd_u64(B + 16 + ch * 16) : 0;',
     '        L->sent = (uint32_t)rd_u64(B + 16 + ch * 16);'),
    ('frames: recv from send slot', None,
     '        L->recv = ch < nch ? (uint32_t)rd_u64(B + 16 + ch * 16 + 8) : 0;',
     '        L->recv = ch < nch ? (uint32_t)rd_u64(B + 16 + ch * 16) : 0;'),
    ('frames: duplicate before range', None,
     '  if (bad_range) return ORC_E_RANGE;\n  if (dup) return ORC_E_DUPLICATE_KEY;',
     '  if (dup) return ORC_E_DUPLICATE_KEY;\n  if (bad_range) return ORC_E_RANGE;'),
    ('frames: count limit off by one', None,
     'if (rd_u64(B + 16 + ch * 16) > 0xFFFFFFFFull ||',
     'if (rd_u64(B + 16 + ch * 16) >= 0xFFFFFFFFull ||'),
    ('hang: seq is minimum over channels', None,
     '        if (s[L].seq > seq) seq = s[L].seq;',
     '        if (ch == 0 || s[L].seq < seq) seq = s[L].seq;'),
    ('hang: entered means not behind by more than one', None,
     '      PQ(q, PAIR_ENTERED) = ((uint64_t)PQ(q, PAIR_SEQ) == seq_max);',
     '      PQ(q, PAIR_ENTERED) = ((uint64_t)PQ(q, PAIR_SEQ) + 1 >= seq_max);'),
    ('hang: idle ignores recv', None,
     '          if (PQ(r2, PAIR_SENT) != PQ(q, PAIR_SENT) || PQ(r2, PAIR_RECV) != PQ(q, PAIR_RECV)) idle_ok = 0;',
     '          if (PQ(r2, PAIR_SENT) != PQ(q, PAIR_SENT)) idle_ok = 0;'),
    ('hang: tree compared as ring', None,
     '    if (T->algo[c] == 1 && T->tree_parent)\n      for (uint32_t q = 0; q < n; ++q) { int32_t par',
     '    if (0)\n      for (uint32_t q = 0; q < n; ++q) { int32_t par'),
    ('hang: sums over first channel only', None,
     '        S += s[L].sent; Rv += s[L].recv;',
     '        if (ch == 0) { S += s[L].sent; Rv += s[L].recv; }'),
]


PIN_FILES = sorted(f for f in os.listdir(os.path.join(ROOT, "tests")) if f.startswith("test_oracle_") and f.endswith(".py"))


def _sandbox(d):
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(d, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests"), os.path.join(d, "tests"), ignore=shutil.ignore_patterns("__pycache__"))
    os.symlink(os.path.join(ROOT, "paper_2605_04478_amd"), os.path.join(d, "paper_2605_04478_amd"))


def _run_pins(d, files):
    return subprocess.run([sys.executable, "-m", "pytest"] + [os.path.join("tests", f) for f in files] +
                          ["-x", "-q", "-p", "no:cacheprovider"], cwd=d, capture_output=True, text=True)


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
    """Every mutant is built and tried in a sandbox of its own, several at a time."""
    from concurrent.futures import ThreadPoolExecutor
    src = open(os.path.join(ROOT, "oracle", "ccld_oracle.c")).read()
    base = str(tmp_path_factory.mktemp("mutants"))

    def one(i):
        what, pin_file, old, new = MUTATIONS[i]
        if src.count(old) != 1:
            return ("pattern", src.count(old))
        d = os.path.join(base, "m%d" % i)
        os.mkdir(d)
        _sandbox(d)
        open(os.path.join(d, "oracle", "ccld_oracle.c"), "w").write(src.replace(old, new))
        p = _run_pins(d, [pin_file] if pin_file else PIN_FILES)
        shutil.rmtree(d, ignore_errors=True)
        return ("ran", p.returncode, p.stdout[-600:], p.stderr[-300:])

    with ThreadPoolExecutor(max_workers=max(1, min(8, os.cpu_count() or 1))) as ex:
        return list(ex.map(one, range(len(MUTATIONS))))


@pytest.mark.parametrize("i", range(len(MUTATIONS)), ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(verdicts, i):
    v = verdicts[i]
    assert v[0] == "ran", "the text to replace must occur exactly once in the oracle (found %s times)" % (v[1],)
    assert v[1] == 1, (MUTATIONS[i][0], v[2], v[3])          # pytest's exit status 1: a test failed


def test_the_unchanged_copy_passes(tmp_path):
    """The sandbox itself is sound: with the oracle's own source every pin file passes there."""
    d = str(tmp_path)
    _sandbox(d)
    p = _run_pins(d, PIN_FILES)
    assert p.returncode == 0, (p.stdout[-800:], p.stderr[-400:])
