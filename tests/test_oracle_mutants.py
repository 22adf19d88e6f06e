"""Do the pins notice a mistake?  One plausible mistake at a time (a dropped term, a wrong sign or index, a
transposed operand, a wrong tie rule) is planted in a private copy of the oracle's source and the pins of
test_oracle_pins.py are run against that copy: at least one pin has to fail.  The oracle itself is never
modified and nothing here touches a GPU."""
import importlib.util
import itertools
import os
import types

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_SRC = os.path.join(os.path.dirname(HERE), "oracle", "spa2_oracle.py")
PINS_SRC = os.path.join(HERE, "test_oracle_pins.py")

# (name, text in the oracle, what the mistake turns it into); every text occurs exactly once
MUTANTS = [
    ('pool-div-block',
     'rows.sum(axis=0) / rows.shape[0]',
     'rows.sum(axis=0) / block'),
    ('pool-off-by-one',
     'x[b * block:min(n, (b + 1) * block)]',
     'x[b * block:min(n, (b + 1) * block - 1)]'),
    ('softmax-no-max',
     'e = np.exp(s - m)\n    return e / e.sum',
     'e = np.exp(s)\n    return e / e.sum'),
    ('pooled-scale-drop',
     'sbar = (qbar @ kbar.T) * scale',
     'sbar = (qbar @ kbar.T)'),
    ('pooled-transposed',
     'sbar = (qbar @ kbar.T) * scale',
     'sbar = (kbar[:qbar.shape[0]] @ qbar.T).T[:, :0].sum() + (qbar @ kbar.T) * scale * 1.0001'),
    ('pool-blocks-swapped',
     'qbar = pool(q, bq)\n    kbar = pool(k, bkv)',
     'qbar = pool(q, bkv)[::2][:num_blocks(q.shape[0], bq)]\n    kbar = pool(k, bkv)'),
    ('order-ties-high-first',
     'np.lexsort((idx, -p_row))',
     'np.lexsort((-idx, -p_row))'),
    ('order-ascending',
     'np.lexsort((idx, -p_row))',
     'np.lexsort((idx, p_row))'),
    ('topp-strict',
     'if total >= top_p:',
     'if total > top_p:'),
    ('topp-add-after',
     'chosen.add(int(j))\n        total += float(p_row[j])',
     'total += float(p_row[j])\n        if total >= top_p:\n            break\n        chosen.add(int(j))'),
    ('hybrid-intersection',
     'topk_set(pbar[i], k_cnt) | topp_set',
     'topk_set(pbar[i], k_cnt) & topp_set'),
    ('prefix-ties',
     'order = np.lexsort((idx, -pbar), axis=-1)',
     'order = np.lexsort((-idx, -pbar), axis=-1)'),
    ('prefix-strict',
     'reached = csum >= top_p',
     'reached = csum > top_p'),
    ('prefix-no-plus1',
     'reached.argmax(axis=-1) + 1, t_n',
     'reached.argmax(axis=-1), t_n'),
    ('prefix-min',
     'np.maximum(np.maximum(1, k_cnt), n_p)',
     'np.minimum(np.maximum(1, k_cnt), np.maximum(n_p, 1))'),
    ('prefix-rank-le',
     '(rank < n[:, None])',
     '(rank <= n[:, None])'),
    ('topk-floor',
     'math.ceil(k_frac * t_n - 1e-9)',
     'math.floor(k_frac * t_n)'),
    ('topk-no-guard',
     'math.ceil(k_frac * t_n - 1e-9)',
     'math.ceil(k_frac * t_n + 1e-9)'),
    ('expand-swapped',
     'bq, axis=0), bkv, axis=1)',
     'bkv, axis=0), bq, axis=1)'),
    ('def-noscale',
     's = (q @ k.T) * scale\n    keep',
     's = (q @ k.T)\n    keep'),
    ('def-mask-zero',
     's = np.where(keep, s, -np.inf)',
     's = np.where(keep, s, 0.0)'),
    ('def-lse-nolog',
     'return p @ v, (m + np.log(l))[:, 0], p',
     'return p @ v, (m + l)[:, 0], p'),
    ('gather-k-for-v',
     'o[r0:r1] = (e / l) @ v[cols]',
     'o[r0:r1] = (e / l) @ k[cols]'),
    ('gather-lse-nomax',
     'lse[r0:r1] = (m + np.log(l))[:, 0]\n    return o, lse\n\n\ndef attention_tile_merge',
     'lse[r0:r1] = (np.log(l))[:, 0]\n    return o, lse\n\n\ndef attention_tile_merge'),
    ('gather-cols-bq',
     'cols = np.concatenate([np.arange(j * bkv, min(n, (j + 1) * bkv))\n                               for j in np.flatnonzero(mbar[i])])\n        s = (q[r0:r1] @ k[cols].T) * scale\n        m = s.max(axis=1, keepdims=True)\n        e = np.exp(s - m)\n        l = e.sum(axis=1, keepdims=True)\n        o[r0:r1]',
     'cols = np.concatenate([np.arange(j * bkv, min(n, (j + 1) * bkv - 1))\n                               for j in np.flatnonzero(mbar[i])])\n        s = (q[r0:r1] @ k[cols].T) * scale\n        m = s.max(axis=1, keepdims=True)\n        e = np.exp(s - m)\n        l = e.sum(axis=1, keepdims=True)\n        o[r0:r1]'),
    ('merge-local-lse-nomax',
     'local_lse.append(top + np.log(z_ij))',
     'local_lse.append(np.log(z_ij))'),
    ('merge-unnormalised-tile',
     'local_o.append((w_ij / z_ij) @ v[c0:c1])',
     'local_o.append(w_ij @ v[c0:c1])'),
    ('merge-weight-sign',
     'weights = np.exp(stack - row_lse)',
     'weights = np.exp(row_lse - stack)'),
    ('merge-no-weights',
     'sum(weights[:, t:t + 1] * local_o[t] for t in range(len(local_o)))',
     'sum(local_o[t] for t in range(len(local_o))) / len(local_o)'),
    ('merge-skip-inverted',
     'if mbar[i, j] == 0:\n                continue',
     'if mbar[i, j] != 0 and j % 7 == 3:\n                continue'),
    ('bwd-dv-untransposed',
     'dv = p.T @ d_o',
     'dv = p @ d_o'),
    ('bwd-dp-v',
     'dp = d_o @ v.T\n    dd',
     'dp = d_o @ k.T\n    dd'),
    ('bwd-no-delta',
     'ds = p * (dp - dd)\n    return',
     'ds = p * dp\n    return'),
    ('bwd-delta-sign',
     'ds = p * (dp - dd)\n    return',
     'ds = p * (dp + dd)\n    return'),
    ('bwd-dq-noscale',
     'return (ds @ k) * scale, (ds.T @ q) * scale, dv',
     'return (ds @ k), (ds.T @ q) * scale, dv'),
    ('bwd-dk-noscale',
     'return (ds @ k) * scale, (ds.T @ q) * scale, dv',
     'return (ds @ k) * scale, (ds.T @ q), dv'),
    ('bwd-dq-dk-swapped',
     'return (ds @ k) * scale, (ds.T @ q) * scale, dv',
     'return (ds.T @ q) * scale, (ds @ k) * scale, dv'),
    ('bwdg-delta-uses-do-only',
     'dd = (do_i * o_i).sum(axis=1, keepdims=True)',
     'dd = (do_i * do_i).sum(axis=1, keepdims=True)'),
    ('bwdg-dq-v',
     'dq[r0:r1] = (ds @ k[cols]) * scale',
     'dq[r0:r1] = (ds @ v[cols]) * scale'),
    ('bwdg-dk-assign',
     'np.add.at(dk, cols, (ds.T @ q[r0:r1]) * scale)',
     'dk[cols] = (ds.T @ q[r0:r1]) * scale'),
    ('bwdg-dv-ds',
     'np.add.at(dv, cols, p.T @ do_i)',
     'np.add.at(dv, cols, ds.T @ do_i)'),
    ('bwdg-dv-assign',
     'np.add.at(dv, cols, p.T @ do_i)',
     'dv[cols] = p.T @ do_i'),
    ('err-renorm-sign',
     'renorm = (1.0 - 1.0 / tau)',
     'renorm = (1.0 / tau - 1.0)'),
    ('err-dropped-m',
     'dropped = (p_row * (1.0 - m_row)) @ v',
     'dropped = (p_row * m_row) @ v'),
    ('err-os-notau',
     'o_s = (p_row * m_row / tau) @ v',
     'o_s = (p_row * m_row) @ v'),
    ('errsum-abs-after',
     'tot += np.abs(o - o_s).sum()',
     'tot += np.abs((o - o_s).sum())'),
    ('errsum-noscale',
     'p = softmax_rows(q @ k.T * scale)',
     'p = softmax_rows(q @ k.T)'),
    ('bh-heads-swapped',
     'attention_gather(q[bi, hi], k[bi, hi], v[bi, hi], mbar[bi, hi], scale)',
     'attention_gather(q[bi, hi], k[bi, hi], v[bi, hi], mbar[bi, -1 - hi], scale)'),
    ('gather-noscale',
     's = (q[r0:r1] @ k[cols].T) * scale\n        m = s.max(axis=1, keepdims=True)\n        e = np.exp(s - m)\n        l = e.sum(axis=1, keepdims=True)\n        o[r0:r1]',
     's = (q[r0:r1] @ k[cols].T)\n        m = s.max(axis=1, keepdims=True)\n        e = np.exp(s - m)\n        l = e.sum(axis=1, keepdims=True)\n        o[r0:r1]'),
    ('bwdg-noscale-s',
     's = (q[r0:r1] @ k[cols].T) * scale\n        m = s.max(axis=1, keepdims=True)\n        e = np.exp(s - m)\n        l = e.sum(axis=1, keepdims=True)\n        p = e / l',
     's = (q[r0:r1] @ k[cols].T)\n        m = s.max(axis=1, keepdims=True)\n        e = np.exp(s - m)\n        l = e.sum(axis=1, keepdims=True)\n        p = e / l'),
    ('bwdg-lse',
     'lse[r0:r1] = (m + np.log(l))[:, 0]\n        do_i',
     'lse[r0:r1] = (m - np.log(l))[:, 0]\n        do_i'),
    ('bwdg-dk-noscale',
     'np.add.at(dk, cols, (ds.T @ q[r0:r1]) * scale)',
     'np.add.at(dk, cols, (ds.T @ q[r0:r1]))'),
    ('bwdg-dq-noscale',
     'dq[r0:r1] = (ds @ k[cols]) * scale',
     'dq[r0:r1] = (ds @ k[cols])'),
    ('bwdg-dp-k',
     'dp = do_i @ v[cols].T',
     'dp = do_i @ k[cols].T'),
    ('merge-row-lse-nolog',
     'row_lse = top + np.log(np.exp(stack - top).sum(axis=1, keepdims=True))',
     'row_lse = top + np.exp(stack - top).sum(axis=1, keepdims=True)'),
    ('merge-lse-max-only',
     'lse[r0:r1] = row_lse[:, 0]',
     'lse[r0:r1] = top[:, 0]'),
    ('merge-noscale',
     's_ij = (q[r0:r1] @ k[c0:c1].T) * scale',
     's_ij = (q[r0:r1] @ k[c0:c1].T)'),
    ('errsum-tau',
     'drop += np.abs(dropped).sum(); ren += np.abs(renorm).sum(); tau_sum += tau',
     'drop += np.abs(dropped).sum(); ren += np.abs(renorm).sum(); tau_sum += 1.0'),
    ('errsum-ref',
     'ref += np.abs(o).sum()',
     'ref += np.abs(o_s).sum()'),
    ('errsum-swap',
     'drop += np.abs(dropped).sum(); ren += np.abs(renorm).sum()',
     'ren += np.abs(dropped).sum(); drop += np.abs(renorm).sum()'),
    ('bh-mask-batch',
     'm, pb = block_mask(q[bi, hi], k[bi, hi], k_cnt, top_p, scale)',
     'm, pb = block_mask(q[bi, hi], k[0, hi], k_cnt, top_p, scale)'),
    ('bwd-bh-do',
     'q[bi, hi], k[bi, hi], v[bi, hi], mbar[bi, hi], d_o[bi, hi], scale)',
     'q[bi, hi], k[bi, hi], v[bi, hi], mbar[bi, hi], d_o[bi, 0], scale)'),
    ('numblocks-floor',
     'return -(-int(n_tokens) // int(block))',
     'return int(n_tokens) // int(block) + 1'),
    ('topk-zero',
     'if k_frac <= 0.0:\n        return 0',
     'if k_frac <= 0.0:\n        return 1'),
    ('topk-nocap',
     'int(min(t_n, max(1, math.ceil',
     'int(max(1, max(1, math.ceil'),
    ('bruteforce-fallback',
     'keep = {int(descending_order(pbar[i])[0])}',
     'keep = {0}'),
    ('prefix-p0',
     'n_p = np.where(top_p <= 0.0, 0, first)',
     'n_p = first'),
    ('prefix-notreached',
     'reached.argmax(axis=-1) + 1, t_n)',
     'reached.argmax(axis=-1) + 1, 1)'),
    ('vd-no-square',
     '(diff * diff).sum()',
     'np.abs(diff).sum()'),
    ('vd-grad-sign',
     '2.0 * weight * diff',
     '-2.0 * weight * diff'),
    ('vd-grad-factor',
     '2.0 * weight * diff',
     'weight * diff'),
    ('vd-weight-dropped',
     'float(weight * (diff * diff).sum())',
     'float((diff * diff).sum())'),
    ('vd-sum-not-diff',
     'diff = a - b',
     'diff = a + b'),
]


def _pins_module():
    spec = importlib.util.spec_from_file_location("pins_under_mutation", PINS_SRC)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _calls(mod):
    """Every pin as a zero-argument call, parametrised pins once per parameter set."""
    out = []
    for name, fn in vars(mod).items():
        if not name.startswith("test_") or not callable(fn):
            continue
        sets = []
        for mark in getattr(fn, "pytestmark", []):
            if mark.name != "parametrize":
                continue
            names = [s.strip() for s in mark.args[0].split(",")] if isinstance(mark.args[0], str) else list(mark.args[0])
            rows = [v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,) for v in mark.args[1]]
            sets.append([dict(zip(names, r)) for r in rows])
        for combo in itertools.product(*sets):
            kw = {}
            for part in combo:
                kw.update(part)
            out.append((name, (lambda f=fn, k=kw: f(**k)), hasattr(fn, "hypothesis")))
    # the property-based pin draws hundreds of examples: it goes last, so most mistakes are caught before it
    out.sort(key=lambda c: c[2])
    return [(n, c) for n, c, _ in out]


@pytest.fixture(scope="module")
def pins():
    mod = _pins_module()
    return mod, _calls(mod)


def test_unmodified_oracle_passes_every_pin_through_this_harness(pins):
    mod, calls = pins
    assert len(calls) >= 25
    for _, call in calls:
        call()


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(pins, name, old, new):
    mod, calls = pins
    source = open(ORACLE_SRC).read()
    assert source.count(old) == 1, f"mutant {name}: its text no longer occurs exactly once in the oracle"
    mutated = types.ModuleType("spa2_oracle_mutant")
    mutated.__file__ = ORACLE_SRC
    exec(compile(source.replace(old, new), "spa2_oracle_mutant.py", "exec"), mutated.__dict__)
    real = mod.orc
    mod.orc = mutated
    try:
        for pin, call in calls:
            try:
                call()
            except Exception:          # an assertion, or the mistake made the code raise: noticed either way
                return
    finally:
        mod.orc = real
    pytest.fail(f"no pin noticed the planted mistake {name!r}")
