"""GPU parity on random problems under random plan options.

The other GPU tests enumerate shapes and options by hand; this one draws them: ranks 2-8, 2^10 to
2^20 elements, both element sizes, forced classes, explicit tiles (with and without line-aligned
windows), the large-tensor form, cache policies, walk orders, workgroup sizes, LDS buffering,
pairs, input windows, the model-based selector, pointers at odd element offsets, plain and
accumulating execution.  An option set the planner rejects (TPERM_ERR_KERNEL) is skipped; one it
accepts must reproduce the oracle bit for bit and leave the guard bands alone.  Seeded, so a
failure names a case that can be replayed.
"""
import math

import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import binding as B

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

GUARD = 256
FILL = -7


def _draw_problem(rng):
    rank = int(rng.integers(2, 9))
    budget = int(2 ** rng.uniform(10, 20))
    dims, vol = [], 1
    for z in range(rank):
        hi = max(2, int((budget / vol) ** (1.0 / (rank - z)) * 2))
        d = int(rng.integers(1, hi + 1))
        dims.append(d)
        vol *= d
    if rng.random() < 0.3:      # an even extent: pairs become possible
        z = int(rng.integers(0, rank))
        dims[z] = max(2, dims[z] // 2 * 2)
    if rng.random() < 0.2:      # a line-aligned extent
        dims[int(rng.integers(0, rank))] = int(rng.choice([16, 32, 64, 128]))
    return dims, [int(p) for p in rng.permutation(rank)], int(rng.choice([4, 8]))


def _draw_options(rng, rank, elem):
    kw = {}
    mode = int(rng.integers(0, 5))
    if mode == 1:
        kw["kernel_class"] = int(rng.choice([B.KERNEL_TILED, B.KERNEL_PACKED, B.KERNEL_ROWCOPY, B.KERNEL_NAIVE]))
    if mode >= 2:
        kw.update(kernel_class=B.KERNEL_PACKED, m=int(rng.integers(1, rank + 1)), k=int(rng.integers(1, rank + 1)),
                  tile_in=int(rng.integers(0, 70)), tile_out=int(rng.integers(0, 70)))
        if rng.random() < 0.5:  # a tile that line-aligned windows can take
            kw.update(tile_out=int(128 // elem * rng.integers(1, 4)), k=1, align_out=2)
    for name, chance, draw in [
            ("large", 0.4, lambda: 1), ("cache_policy", 0.5, lambda: int(rng.integers(1, 5))),
            ("grid_mode", 0.3, lambda: int(rng.choice([-1, 1, 2, 4, 7, 9]))), ("vec2", 0.3, lambda: int(rng.integers(0, 3))),
            ("threads", 0.2, lambda: int(rng.choice([64, 256]))), ("lds_buffers", 0.2, lambda: int(rng.integers(1, 3))),
            ("loads_first", 0.2, lambda: int(rng.integers(1, 3))), ("align_out", 0.2, lambda: int(rng.integers(1, 3))),
            ("window_in", 0.2, lambda: int(rng.integers(-1, 12))), ("window_out", 0.2, lambda: int(rng.integers(1, 12))),
            ("tile_order", 0.2, lambda: int(rng.integers(1, 3))), ("lds_pad", 0.2, lambda: int(rng.integers(0, 8))),
            ("selector", 0.2, lambda: 1)]:
        if rng.random() < chance:
            kw[name] = draw()
    return kw


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_problems_under_random_options(seed):
    rng = np.random.default_rng(seed)
    stream = torch.cuda.current_stream().cuda_stream
    ran = rejected = 0
    for it in range(400):
        dims, perm, elem = _draw_problem(rng)
        vol = math.prod(dims)
        if vol < 2 or vol > (1 << 21):
            continue
        kw = _draw_options(rng, len(dims), elem)
        where = f"seed {seed} draw {it}: dims={dims} perm={perm} elem={elem} options={kw}"
        try:
            plan = B.tperm_plan_create_ex(dims, perm, elem, **kw)
        except B.TpermError as e:
            assert e.status == B.ERR_KERNEL, where
            rejected += 1
            continue
        info = plan.describe()
        in_off, out_off = int(rng.integers(0, 4)), int(rng.integers(0, 40))
        if info.vec2 and not info.align_out and kw.get("vec2") == 2:
            in_off, out_off = in_off // 2 * 2, out_off // 2 * 2     # pairs forced into the plan itself: aligned pointers
        sign = np.int64 if elem == 8 else np.int32
        dt = torch.int64 if elem == 8 else torch.int32
        abuf = torch.zeros(vol + 8, dtype=dt, device="cuda")
        a = abuf[in_off:in_off + vol]
        obuf = torch.full((vol + 2 * GUARD + 64,), FILL, dtype=dt, device="cuda")
        o = obuf[GUARD + out_off:GUARD + out_off + vol]
        accumulate = rng.random() < 0.25
        if accumulate:
            # small integers as floating point: the one addition per element is exact
            ftype = np.float64 if elem == 8 else np.float32
            av = rng.integers(0, 1000, size=vol).astype(ftype)
            bv = rng.integers(0, 1000, size=vol).astype(ftype)
            a.copy_(torch.from_numpy(av.view(sign)))
            o.copy_(torch.from_numpy(bv.view(sign)))
            ref = (oracle.transpose(av, dims, perm) + bv).view(sign)
            run = B.tperm_execute_accumulate
        else:
            av = rng.integers(-2 ** 63, 2 ** 63, size=vol, dtype=np.int64).astype(sign)   # raw bits, high half included
            a.copy_(torch.from_numpy(av))
            ref = oracle.transpose(av, dims, perm)
            run = B.tperm_execute
        try:
            run(plan, a.data_ptr(), o.data_ptr(), stream)
        except B.TpermError as e:
            # forms that have no accumulating kernel, or pairs with a pointer they cannot take
            assert e.status in (B.ERR_KERNEL, B.ERR_ALIGN), where
            rejected += 1
            continue
        torch.cuda.synchronize()
        got = o.cpu().numpy()
        bad = np.nonzero(got != ref)[0]
        assert bad.size == 0, f"{where} accumulate={accumulate} offsets={in_off},{out_off}: {bad.size} wrong elements, first {bad[:4]}; plan={B.info_dict(info)}"
        assert bool((obuf[:GUARD + out_off] == FILL).all()) and bool((obuf[GUARD + out_off + vol:] == FILL).all()), \
            f"{where}: wrote outside the output; plan={B.info_dict(info)}"
        ran += 1
    assert ran >= 150, (ran, rejected)
