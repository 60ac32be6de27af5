"""Plants one mistake at a time in a COPY of the oracle and checks that the CPU pins notice.

Not collected by pytest (it takes a quarter of an hour): run it by hand with
    python tests/planted_mistakes.py [group ...]
It copies oracle/, tests/, workloads.py and the package into a scratch directory, rewrites one expression of
one oracle source there, and runs the pin tests of that oracle in the copy -- without the tests that compare
the product with the oracle, which would notice a wrong oracle too but are no pins.  A mistake that the pins
do not notice is a hole in them, unless it is listed here as equivalent (it changes no result).  Exit status 1
if a mistake that should be caught survives.  Nothing here touches the GPU or the product's sources.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EQUIVALENT = "equivalent"

# group -> (oracle source, pin tests, tests left out because they involve the product, [(old, new, note)])
GROUPS = {
    "c_oracle": ("oracle/r2_oracle.c", "tests/test_oracle_partition.py tests/test_oracle_reduce.py", [], [
        ("u += 0x7fffu + kept_lsb;", "u += 0x8000u;", "ties rounded up instead of to even"),
        ("u += 0x7fffu + kept_lsb;", "u += 0;", "truncation instead of rounding"),
        ("e[c] = ((fail_mask >> c) & 1u) ? 0u : weights[c];", "e[c] = weights[c];", "failed channels keep their weight"),
        ("if (P == W)\n", "if (P == W && c > 0)\n", EQUIVALENT + ": P = W at channel 0 means W = 0, which is refused before"),
        ("if (P == W)\n", "if (0)\n", "no special case once every healthy channel has been served"),
        ("(((unsigned __int128)U * P) / W);", "(((unsigned __int128)U * P + W - 1) / W);", "ceiling instead of floor"),
        ("(start + 2 * R - j) % R", "(start + j) % R", "ring chunk index runs the wrong way"),
        ("(phases == R2O_PHASE_AG) ? r + 1 : r;", "r;", "all-gather alone starts at the wrong chunk"),
        ("uint32_t peer = (r + R - 1) % R;", "uint32_t peer = (r + 1) % R;", "receive from the successor"),
        ("STAGE_PTR((j - 1) & 1, peer, l, k)", "STAGE_PTR(j & 1, peer, l, k)", "wrong stage parity"),
        ("op = (j <= R - 1) ? R2O_OP_SUM : R2O_OP_COPY;", "op = (j <= R) ? R2O_OP_SUM : R2O_OP_COPY;", "one reducing step too many"),
        ("((r + R - c) % R) + 1 : R;", "((c + R - r) % R) + 1 : R;", "reduce-scatter definition: terms counted the wrong way round"),
        ("uint32_t owner = (c + R - 1) % R;", "uint32_t owner = c;", "all-gather definition: wrong owner"),
        ("if (ep[i].t_start <= t) cur", "if (ep[i].t_start < t) cur", "an epoch starts one transmission late"),
        ("(uint64_t)l * T_slab + j - 1);", "(uint64_t)l * T_slab + j);", "the reader uses its own transmission's table"),
        ("float acc = ((const float *)in[c])[base + i];", "float acc = ((const float *)in[(c + 1) % R])[base + i];", "the fold starts at the wrong rank"),
    ]),
    "c_failover_and_relay": ("oracle/r2_oracle.c",
                             "tests/test_oracle_rollback.py tests/test_oracle_split.py tests/test_oracle_inflight.py",
                             ["tests/test_oracle_split.py::test_product_planner_matches_oracle",
                              "tests/test_oracle_split.py::test_partial_elems_follow_the_share_and_fit_both_rings"], [
        ("int newly = ((mask_after >> f) & 1u) && !((mask_before >> f) & 1u);", "int newly = ((mask_after >> f) & 1u);", "channels that were down before get a plan too"),
        ("int r = r2o_partition(weights, mask_after, C, len, align, row);", "int r = r2o_partition(weights, mask_before, C, len, align, row);", "shared out over the old survivors"),
        ("uint64_t len = off[f + 1] - off[f];\n        if (!newly", "uint64_t len = off[f + 1];\n        if (!newly", "slice length taken for its end"),
        ("if ((mask_before & ~mask_after) != 0) return R2O_INVALID;", "if (0) return R2O_INVALID;", "a recovery accepted as a rollback"),
        ("memcpy(out_stage[c], (relay ? relay : v) + out_off[c], len);", "memcpy(out_stage[c], v + out_off[c], len);", "the relay step forwards the sum"),
        ("if (op == R2O_OP_SUM || op == R2O_OP_SUM_FORWARD) {", "if (op == R2O_OP_SUM) {", "the relay step does not add"),
        ("uint64_t *row = plan + (uint64_t)f * (C + 1);", "uint64_t *row = plan + (uint64_t)f * C;", "plan rows overlap"),
    ]),
    "inflight": ("oracle/inflight.py", "tests/test_oracle_inflight.py", [], [
        ("t0 + 1 if fl else t0", "t0 if fl else t0", "the struck transmission already uses the new table"),
        ("t0 + 1 if fl else t0", "t0 + 2 if fl else t0", "the new table comes one transmission late"),
        ("e[0] < shifted[i + 1][0]", "e[0] <= shifted[i + 1][0]", "an epoch overtaken by an in-flight one before it still cuts a table"),
        ("o.rollback_plan(log[k], epochs[i][2]", "o.rollback_plan(log[k - 1], epochs[i][2]", "the plan reads the row before"),
        ("o.rollback_plan(log[k], epochs[i][2], epochs[i - 1][1], epochs[i][1]", "o.rollback_plan(log[k], epochs[i - 1][2], epochs[i - 1][1], epochs[i][1]", "the plan shares by the old weights"),
        ("epochs[i][2], epochs[i - 1][1], epochs[i][1], align)", "epochs[i][2], epochs[i][1], epochs[i][1], align)", "nothing is newly failed"),
        ("epochs[i][2], epochs[i - 1][1], epochs[i][1], align)", "epochs[i][2], epochs[i - 1][1], epochs[i - 1][1] | epochs[i][1], align)", EQUIVALENT + ": an in-flight epoch's mask contains its predecessor's"),
        ("if fl and (epochs[i - 1][1] & ~epochs[i][1])", "if fl and (epochs[i][1] & ~epochs[i - 1][1])", "failures refused, recoveries accepted"),
        ("if fl and k < log.shape[0]:", "if fl and k + 1 < log.shape[0]:", "no plan for the last transmission"),
        ("return [e for i, e in enumerate(shifted) if i + 1 == len(shifted) or e[0] < shifted[i + 1][0]]", "return shifted", "an overtaken epoch still cuts tables"),
    ]),
    "recursive": ("oracle/recursive.py", "tests/test_oracle_recursive.py",
                  ["test_host_planner_matches_oracle", "test_host_planner_on_the_share_rules_corner_cases",
                   "test_segments_follow_the_shares_and_fit_the_rings", "test_host_selector_ties_go_to_the_shallower_plan",
                   "test_host_planner_rejects_bad_arguments"], [
        ("start = excl[-1] + 1 if excl else 0", "start = excl[0] + 1 if excl else 0", "the ring starts after the first rank left out"),
        ("return bridge_rerank(base, rails)[0]", "return base", "no re-ranking"),
        ("u = [1 / f[k] if k <= j else 1 / f[j] for k in range(L)]", "u = [1 / f[k] if k < j else 1 / f[j] for k in range(L)]", EQUIVALENT + ": both branches give 1/f[j] at k = j"),
        ("if best is None or t < best[0]:", "if best is None or t <= best[0]:", "ties go to the later balance level"),
        ("t = tau * (1 + 1 / f[j])", "t = tau * (1 + 1 / f[-1])", "broadcast time of the wrong level"),
        ("for j in range(1, L):", "for j in range(L - 1, L):", "all rings always finish together"),
        ("for j in range(1, L):", "for j in range(1, 2):", "only the two lowest rings ever finish together"),
        ("return n_members + 2 * m - 1", "return n_members + 2 * m", "one hop too many"),
        ("red.append(2 * (p - 1) * alpha + ring_factor(p) * t)", "red.append((p - 1) * alpha + ring_factor(p) * t)", "half the ring's latency"),
        ("bc.append(hops(n_ranks, len(lv.members)) * alpha + t)", "bc.append(hops(n_ranks, len(lv.members)) * alpha + ring_factor(p) * t)", "ring factor on the broadcast"),
        ("return max(red) + max(bc)", "return max(red + bc)", "broadcast overlapped with the reductions"),
        ("return max(red) + max(bc)", "return sum(red) + max(bc)", "reductions one after the other"),
        ("key=lambda i: (times[i], i)", "key=lambda i: (times[i], -i)", "ties go to the deeper plan"),
        ("granule = n_slabs * (p * n_ranks // gcd(p, n_ranks)) * per16", "granule = n_slabs * p * per16", "segments fit their own ring only"),
        ("out[k] = int(levels[k].share * n_elems) // granule * granule", "out[k] = -(-int(levels[k].share * n_elems) // granule) * granule", "segments rounded up"),
        ('[(r, "take") for r in excl]', '[(r, "take") for r in reversed(excl)]', "the result is taken in descending order"),
        ('[(r, "gather") for r in excl] + [(r, "member") for r in level.order]', '[(r, "gather") for r in excl] + [(r, "member") for r in level.members]', "the chain ignores the ring's order"),
        ("for w in list(level.order) + excl:", "for w in excl + list(level.order):", "ranks left out are asked to relay first"),
        ("return ((fail_masks[a] | fail_masks[b]) & full) != full", "return ((fail_masks[a] & fail_masks[b]) & full) != full", "linked if either end has a channel"),
        ("if w not in (u, v) and linked(u, w) and linked(w, v):", "if w not in (u, v) and linked(u, w):", "a relay linked to one end only"),
        ("for r in lv.order], dtype, n_slabs, o.PHASE_AR)[0]", "for r in lv.members], dtype, n_slabs, o.PHASE_AR)[0]", "definition folds in rank order, not ring order"),
        ("for r in excl[1:]:\n                    acc = _add(np.ascontiguousarray(inputs[r][lo:hi]), acc, dtype)", "for r in excl[1:]:\n                    acc = _add(acc, np.ascontiguousarray(inputs[r][lo:hi]), dtype)", EQUIVALENT + ": one addition is commutative"),
        ("op = o.OP_SUM if i == last_member else o.OP_SUM_FORWARD", "op = o.OP_SUM_FORWARD", "the last member relays instead of sending its result"),
        ("op = o.OP_SUM if i == last_member else o.OP_SUM_FORWARD", "op = o.OP_SUM", "members forward their sums"),
        ("fail_masks[visits[i][0]] | fail_masks[visits[i + 1][0]], nbytes, align)", "fail_masks[visits[i][0]], nbytes, align)", "a hop is cut by the sender only"),
        ("s_in = stage[(i + 1) & 1] if i else None", "s_in = stage[i & 1] if i else None", "wrong stage parity in the chain"),
        ("return rl.ring_bandwidth(weights, [fail_masks[r] for r in order])", "return min(own_bandwidth(weights, fail_masks[r]) for r in order)", "a ring as fast as its slowest member, whatever its links"),
        ("return Level(list(members), union, bw, bw - prev_bw, Fraction(0), order)", "return Level(list(members), union, bw, bw, Fraction(0), order)", "a level counts its whole bandwidth as added"),
        ("rest = [r for r in members if own[r] > lo]", "rest = [r for r in members if r != min(members, key=lambda q: (own[q], q))]", "equally slow ranks leave one by one"),
        ("if len(rest) < 2:", "if len(rest) < 3:", "no ring of two"),
        ("rl.static_epochs(weights, [fail_masks[r] for r in lv.order])", "rl.static_epochs(weights, [lv.fail_mask for r in lv.order])", "one table for the whole level ring"),
        ("local = np.empty_like(segs[r])", "pass", "a relay overwrites its own segment"),
    ]),
    "split": ("oracle/split.py", "tests/test_oracle_split.py",
              ["test_product_planner_matches_oracle", "test_partial_elems_follow_the_share_and_fit_both_rings"], [
        ("return Fraction(2 * (p - 1), p)", "return Fraction(2 * (p - 1), p + 1)", "ring factor"),
        ("t1 = a * (1 - Y) / (1 - X)", "t1 = a * (1 - Y) / X", "global ring at the wrong bandwidth"),
        ("t2 = b * Y / X ", "t2 = a * Y / X ", "partial ring with the global ring's factor"),
        ("t3 = Y / X ", "t3 = b * Y / X ", "ring factor on the broadcast"),
        ("return max(t1, t2) + t3", "return max(t1, t2 + t3)", "broadcast overlapped with the global ring"),
        ("return a * X / (a * X + b * (1 - X))", "return b * X / (b * X + a * (1 - X))", "balance point with the factors swapped"),
        ("return X + X * (1 - X) / (X + (g * (n - 1) - 1) * n)", "return X + X * (1 - X) / (X + (g * (n - 1)) * n)", "the printed Y* mistyped"),
        ("return Fraction(n * g, 3 * n * g - 2)", "return Fraction(n * g, 3 * n * g - 1)", "threshold"),
        ("return 2 * (1 - Y) + Y", "return 2 * (1 - Y) + 2 * Y", "the degraded server's volume"),
        ("order = [(d + 1 + i) % R for i in range(R - 1)]\n        tails = o.expected", "order = [(d - 1 - i) % R for i in range(R - 1)]\n        tails = o.expected", "definition: partial ring the other way round"),
        ("total = _add(tails[0], xd, dtype)", "total = tails[0]", "definition: the degraded rank's tail left out"),
        ("[(0, degraded_mask, weights)], o.PHASE_AR)", "[(0, 0, weights)], o.PHASE_AR)", "the global ring at full width"),
        ("o.ring_sim(tails, dtype, slabs_partial, n_channels, align, [(0, 0, weights)]", "o.ring_sim(tails, dtype, slabs_partial, n_channels, align, [(0, degraded_mask, weights)]", "the partial ring throttled"),
        ("stage[(k + 1) & 1], t_deg if k == 1 else t_ok,", "stage[(k + 1) & 1], t_ok,", "first healthy rank reads with the full table"),
        ("stage[k & 1], t_deg if last else t_ok, n_channels, cap)", "stage[k & 1], t_ok, n_channels, cap)", "last healthy rank sends with the full table"),
        ("o.OP_SUM if last else o.OP_SUM_FORWARD,", "o.OP_SUM,", "healthy ranks forward their sums"),
        ("o.OP_SUM if last else o.OP_SUM_FORWARD,", "o.OP_SUM_FORWARD,", "the last healthy rank relays"),
        ("o.reduce_copy(d_tail, dtype, o.OP_COPY, stage[(R + 1) & 1], t_deg", "o.reduce_copy(d_tail, dtype, o.OP_COPY, stage[R & 1], t_deg", "the degraded rank reads the wrong parity"),
    ]),
    "rails": ("oracle/rails.py", "tests/test_oracle_rails.py", [], [
        ("return [fail_masks[r] | fail_masks[(r + 1) % R] for r in range(R)]", "return [fail_masks[r] for r in range(R)]", "a link knows its sender only"),
        ("return [fail_masks[r] | fail_masks[(r + 1) % R] for r in range(R)]", "return [fail_masks[r] | fail_masks[(r - 1) % R] for r in range(R)]", "links point backwards"),
        ("return min(link_bandwidth(weights, fail_masks))", "return max(link_bandwidth(weights, fail_masks))", "a ring as fast as its widest link"),
        ("_, m1, w1 = state_at(rank_epochs[(r + 1) % R], t)", "_, m1, w1 = state_at(rank_epochs[(r - 1) % R], t)", "link state from the predecessor"),
        ("return m0 | m1, [min(int(a), int(b))", "return m0 & m1, [min(int(a), int(b))", "a channel down at one end still carries"),
        ("return m0 | m1, [min(int(a), int(b))", "return m0 | m1, [max(int(a), int(b))", "the faster end sets the speed"),
        ("c = (r + first - j) % R", "c = (r + first + j) % R", "chunk index runs the wrong way"),
        ("peer = (r - 1) % R", "peer = (r + 1) % R", "receive from the successor"),
        ("tables[peer, t - 1] if j > 0 else None", "tables[r, t - 1] if j > 0 else None", "read with the own link's table"),
        ("s_out, tables[r, t] if j < J - 1 else None", "s_out, tables[peer, t] if j < J - 1 else None", "write with the predecessor's table"),
        ("op = o.OP_SUM if j <= R - 1 else o.OP_COPY", "op = o.OP_SUM if j < R - 1 else o.OP_COPY", "one reducing step too few"),
        ("stage[(j - 1) & 1, peer, l, k]", "stage[(j - 1) & 1, peer, 0, k]", "every slab reads slab 0's stage"),
        ("t = l * T + j", "t = j", "slabs share their transmissions' tables"),
    ]),
    "rerank": ("oracle/rerank.py", "tests/test_rerank.py",
               ["test_product_on_hand_worked_rings", "test_product_matches_oracle_exhaustive_tiny",
                "test_product_matches_oracle_random", "test_product_rejects_non_permutations"], [
        ("narrowest = min(len(rails[node]) for node in order)", "narrowest = max(len(rails[node]) for node in order)", "the widest node sets the bar"),
        ("if width(u, v) < narrowest:", "if width(u, v) <= narrowest:", "edges that are wide enough are repaired too"),
        ("broken.sort(key=lambda item: (-item[0], item[1]))", "broken.sort(key=lambda item: (item[0], item[1]))", "smallest gap first"),
        ("broken.sort(key=lambda item: (-item[0], item[1]))", "broken.sort(key=lambda item: (-item[0], -item[1]))", "equal gaps against the ring order"),
        ("if n < 3 or order[(at + 1) % n] != v:", "if n < 3:", "a separated pair is repaired again"),
        ("for w in list(order):", "for w in reversed(list(order)):", "bridges tried against the ring order"),
        ("fits = min(width(u, w), width(w, v)) >= narrowest", "fits = max(width(u, w), width(w, v)) >= narrowest", "a bridge wide towards one end only"),
        ("gap_closes = width(before, after) >= narrowest", "gap_closes = True", "the gap a bridge leaves is not looked at"),
        ("order.insert(order.index(u) + 1, w)", "order.insert(order.index(v) + 1, w)", "the bridge goes behind the pair"),
        ("relocations += 1\n                break", "relocations += 1", "every fitting node moves"),
    ]),
    "sendrecv": ("oracle/sendrecv.py", "tests/test_oracle_sendrecv.py", [], [
        ("if e[0] <= t:", "if e[0] < t:", "an epoch starts one message late"),
        ("return [send[(r - 1) % R].copy() for r in range(R)]", "return [send[(r + 1) % R].copy() for r in range(R)]", "definition: from the successor"),
        ("_, mask, weights = state_at(epochs, l)", "_, mask, weights = state_at(epochs, 0)", "the first state for every message"),
        ("bufs = [stage[(r - 1) % R, l, c] for c in range(n_channels)]", "bufs = [stage[r, l, c] for c in range(n_channels)]", "a rank receives its own message"),
    ]),
}


def run_group(name: str) -> int:
    path, tests, left_out, mistakes = GROUPS[name]
    src = open(os.path.join(ROOT, path)).read()
    holes = 0
    for i, (old, new, note) in enumerate(mistakes):
        if src.count(old) < 1:
            print(f"{name} #{i}: the expression to replace is gone: {old!r}", flush=True)
            holes += 1
            continue
        tmp = tempfile.mkdtemp(prefix="planted_")
        try:
            for d in ("oracle", "tests", "paper_2512_25059_amd", "include"):
                shutil.copytree(os.path.join(ROOT, d), os.path.join(tmp, d),
                                ignore=shutil.ignore_patterns("__pycache__", ".pytest_cache"))
            for f in ("workloads.py", "bench.py", "__graft_entry__.py"):
                shutil.copy(os.path.join(ROOT, f), tmp)
            open(os.path.join(tmp, path), "w").write(src.replace(old, new, 1))  # newer than the built oracle: rebuilt on load
            cmd = [sys.executable, "-m", "pytest", *tests.split(), "-q", "-x", "--no-header", "-p", "no:cacheprovider"]
            for t in left_out:
                cmd += ["--deselect", t if "::" in t else f"{tests.split()[0]}::{t}"]
            res = subprocess.run(cmd, cwd=tmp, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        finally:
            shutil.rmtree(tmp, ignore_errors=True)
        caught = res.returncode != 0
        first = next((l for l in res.stdout.splitlines() if l.startswith(("FAILED", "ERROR"))), "")
        expected_alive = note.startswith(EQUIVALENT)
        verdict = "caught" if caught else ("equivalent, alive as expected" if expected_alive else "NOT NOTICED")
        holes += (not caught) and (not expected_alive)
        print(f"{name} #{i:2d} {verdict:30s} {note[:70]:70s} {first[:90]}", flush=True)
    return holes


def main() -> int:
    groups = sys.argv[1:] or list(GROUPS)
    holes = sum(run_group(g) for g in groups)
    print(f"{holes} planted mistake(s) went unnoticed" if holes else "every planted mistake was noticed (or is listed as equivalent)")
    return 1 if holes else 0


if __name__ == "__main__":
    sys.exit(main())
