"""Seeded random cases over the whole argument space of the signature calls, for the
differential test against the CPU oracle (tests/test_random_cases_gpu.py): hash family, universe
size from each range that has a kernel form of its own (powers of two, below 2^26, up to 2^28, up
to p/3, up to p, up to 2^32 for p = 2^61-1, and the edges between them), k from 1 to 1100, b from
1 to 32, row lengths around every tile, chunk and lane-count boundary with empty rows mixed in,
sorted or unsorted rows, extreme indices (0, D-1) and coefficients (0, p-1), a row pitch with pad
bytes, a row_ptr that does not start at 0, each flag, and each entry point (plain, built-in work
space, packed rows).  Inputs only: nothing here evaluates a hash function."""
import numpy as np

P31, P61 = (1 << 31) - 1, (1 << 61) - 1


def pick_D(rng, family):
    if family in (5, 6):
        return 1 << int(rng.integers(1, 33))
    if family == 4:
        return int(rng.integers(1, 3000))
    p = P31 if family in (0, 1) else P61
    top = 31 if family in (0, 1) else 32
    kind = rng.integers(0, 10)
    if kind < 4:
        s = int(rng.integers(0, top + 1))
        D = 1 << s
        if D >= p:
            D = 1 << 30
        return D
    if kind == 4:
        return int(rng.integers(1, 1000))
    if kind == 5:
        return int(rng.integers(1000, 1 << 26))
    if kind == 6:
        return int(rng.integers(1 << 26, 1 << 28))
    if kind == 7:
        return int(rng.integers(1 << 28, P31 // 3 + 2))
    if kind == 8:
        hi = P31 if family in (0, 1) else (1 << 32) + 1
        return int(rng.integers(P31 // 3, hi))
    # edges
    edges = [1, 2, 3, P31 // 3, P31 // 3 + 1, (1 << 28) - 1, (1 << 28) + 1, (1 << 26) + 1, P31 - 1, (1 << 30) + 1]
    if family in (2, 3):
        edges += [(1 << 32) - 1, (1 << 31) + 1, 1 << 32, (1 << 31)]
    return int(edges[int(rng.integers(0, len(edges)))])


def pick_rows(rng, budget_nnz):
    n_rows = int(rng.choice([0, 1, 2, 3, 7, 33, 64, 65, 200, 500, 1100, 2500]))
    kinds = rng.integers(0, 6)
    lens = np.zeros(n_rows, dtype=np.int64)
    for r in range(n_rows):
        c = rng.integers(0, 100)
        if c < 8:
            lens[r] = 0
        elif c < 20:
            lens[r] = rng.integers(1, 5)
        elif c < 60:
            lens[r] = rng.integers(1, 130) if kinds < 4 else rng.integers(200, 600)
        elif c < 85:
            lens[r] = rng.choice([63, 64, 65, 127, 128, 129, 255, 256, 257, 258, 511, 512, 513, 767, 768, 1023, 1024, 1025])
        elif c < 97:
            lens[r] = rng.integers(1000, 5000)
        else:
            lens[r] = rng.choice([8191, 8192, 8193, 12000, 16384, 16385, 40000, 70000])
    # keep the total within budget by clipping from the largest down
    while lens.sum() > budget_nnz and n_rows:
        i = int(np.argmax(lens))
        lens[i] = lens[i] // 2
    return lens


def make_case(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    family = int(rng.choice([0, 0, 0, 1, 1, 2, 2, 3, 5, 6, 4]))
    D = pick_D(rng, family)
    k = int(rng.choice([1, 2, 5, 8, 31, 40, 64, 65, 100, 128, 200, 256, 257, 500, 512, 513, 777, 1000, 1024, 1100]))
    if family == 4:
        k = min(k, 300)
    b = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 8, 8, 12, 16, 16, 24, 31, 32]))
    evals = 2.5e7 if family in (0, 2, 5, 6) else 1.2e7
    lens = pick_rows(rng, max(int(evals / k), 64))
    rp = np.zeros(lens.shape[0] + 1, dtype=np.int64)
    np.cumsum(lens, out=rp[1:])
    nnz = int(rp[-1])
    sorted_rows = bool(rng.integers(0, 2))
    col = rng.integers(0, D, size=nnz, dtype=np.uint64).astype(np.uint32) if nnz else np.zeros(0, np.uint32)
    if nnz and rng.integers(0, 3) == 0:      # extremes
        idx = rng.integers(0, nnz, size=min(nnz, 20))
        col[idx] = np.where(rng.integers(0, 2, size=idx.shape[0]) == 0, 0, D - 1).astype(np.uint32)
    if sorted_rows:
        for r in range(lens.shape[0]):
            col[rp[r]:rp[r + 1]].sort()
    if family == 4:
        ld = k + int(rng.choice([0, 0, 3, 12]))
        params = np.zeros((D, ld), dtype=np.uint32)
        for j in range(k):
            params[:, j] = rng.permutation(D).astype(np.uint32)
    elif family in (5, 6):
        params = rng.integers(0, 1 << 32, size=(k, 2), dtype=np.uint64)
        params[:, 1] |= np.uint64(1)
    else:
        p = P31 if family in (0, 1) else P61
        deg = 2 if family in (0, 2) else 4
        params = rng.integers(0, p, size=(k, deg), dtype=np.uint64)
        if rng.integers(0, 4) == 0:          # extreme coefficients
            params[rng.integers(0, k), :] = 0
            params[rng.integers(0, k), :] = p - 1
            params[rng.integers(0, k), 0] = 0
    sig = (k * b + 7) // 8
    stride = sig + int(rng.choice([0, 0, 0, 1, 3, 16]))
    flags = 0
    f = rng.integers(0, 10)
    if f == 0:
        flags |= 1
    if f == 1 and family in (0, 1, 2):
        flags |= 4
    if f == 2 and family in (0, 1) and nnz * k < 4e6:
        flags |= 2
    entry = 'plain'
    e = rng.integers(0, 10)
    if e < 2 and sorted_rows and family != 4 and lens.shape[0] > 0:
        entry = 'packed'
    elif e < 4:
        entry = 'static'
    base = int(rng.choice([0, 0, 0, 5, 1000])) if entry != 'packed' else 0
    return dict(seed=seed, family=family, D=D, k=k, b=b, rp=rp, col=col, params=params, stride=stride, flags=flags,
                entry=entry, sorted=sorted_rows, base=base)


def describe(c):
    lens = np.diff(c['rp'])
    return 'seed=%d fam=%d D=%d k=%d b=%d rows=%d nnz=%d maxlen=%d stride=%d flags=%d entry=%s sorted=%d base=%d' % (
        c['seed'], c['family'], c['D'], c['k'], c['b'], lens.shape[0], int(c['rp'][-1]), int(lens.max()) if lens.size else 0,
        c['stride'], c['flags'], c['entry'], c['sorted'], c['base'])
