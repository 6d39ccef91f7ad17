"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on
the same seeded inputs.  Bar: schedule and reused outputs bit-exact; computed
attention within max-abs error 1e-2 * max|V| (bf16 operands, fp32 accumulation)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import pab_oracle as orc
from paper_2408_12588_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = 1e-2   # max |gpu - oracle| <= TOL * max|V|
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pab():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2408_12588_amd import pab as mod
    return mod


def rand_qkv(kind, T, S, L, H, D, dtype, seed, scale_rows=0.0):
    wl = W.Workload("case", 1, T, S, L, H, D, dtype, 1, (1, 1, 1), 0, 0, peaked_frac=scale_rows, seed=seed)
    return W.make_qkv(wl, 0, kind, 0)


def assert_close(got: torch.Tensor, want: np.ndarray, v: torch.Tensor, what=""):
    got = got.detach().cpu().double().numpy()
    assert np.isfinite(got).all(), what
    err = np.abs(got - want).max()
    bound = TOL * float(v.abs().max())
    assert err <= bound, "%s: max abs err %.3e > %.3e" % (what, err, bound)
    return err


SHAPES = [
    # kind, T, S, L, H, D, dtype
    (W.SPATIAL, 2, 300, 0, 2, 72, "bf16"),     # 2 query blocks (256 + 44), 5 key blocks, ragged tail
    (W.SPATIAL, 1, 64, 0, 1, 72, "bf16"),      # exactly one key block
    (W.SPATIAL, 1, 65, 0, 3, 72, "bf16"),      # one key past a block edge
    (W.SPATIAL, 3, 513, 0, 3, 72, "bf16"),     # more (batch, head) pairs than one per XCD round
    (W.SPATIAL, 1, 1, 0, 1, 72, "bf16"),       # single token
    (W.SPATIAL, 1, 256, 0, 2, 72, "bf16"),     # one full query block, eight whole key tiles: steady loop, no ragged tile
    (W.SPATIAL, 1, 257, 0, 2, 32, "bf16"),     # one query and one key past the block: a workgroup with a single live row
    (W.SPATIAL, 2, 200, 0, 2, 32, "bf16"),
    (W.SPATIAL, 2, 130, 0, 2, 72, "f32"),
    (W.SPATIAL, 4, 64, 0, 4, 32, "f32"),       # the Tiny configuration's spatial call
    (W.SPATIAL, 1, 512, 0, 260, 72, "bf16"),   # 520 workgroups: the 8 past a full round become split items (4 key groups, combined in LDS)
    (W.SPATIAL, 1, 700, 0, 261, 72, "bf16"),   # ... with a ragged last query block and a ragged last key tile in every key group
    (W.SPATIAL, 1, 520, 0, 264, 32, "f32"),    # ... head dim 32, fp32 rows (staged through registers)
    (W.TEMPORAL, 16, 50, 0, 4, 72, "bf16"),
    (W.TEMPORAL, 17, 37, 0, 3, 72, "bf16"),    # 17 frames: second 16-key half almost empty
    (W.TEMPORAL, 1, 9, 0, 2, 72, "bf16"),      # one frame: identity on V
    (W.TEMPORAL, 4, 64, 0, 4, 32, "f32"),      # Tiny
    (W.TEMPORAL, 32, 11, 0, 2, 72, "bf16"),    # full 32x32 tile
    (W.TEMPORAL, 24, 13, 0, 2, 72, "bf16"),    # last clip length of the 24-row staging variant
    (W.TEMPORAL, 25, 13, 0, 2, 72, "f32"),     # first of the 32-row variant
    (W.TEMPORAL, 33, 7, 0, 2, 72, "bf16"),     # beyond the wavefront-resident kernel: tiled fallback
    (W.TEMPORAL, 5, 300, 0, 16, 72, "f32"),
    (W.TEMPORAL, 16, 33, 0, 2, 32, "bf16"),
    (W.CROSS, 2, 300, 120, 2, 72, "bf16"),
    (W.CROSS, 3, 100, 300, 2, 72, "bf16"),
    (W.CROSS, 1, 70, 1, 2, 72, "bf16"),        # one text key: output = its value
    (W.CROSS, 4, 64, 16, 4, 32, "f32"),        # Tiny
    (W.CROSS, 2, 129, 64, 1, 72, "f32"),
    (W.CROSS, 5, 101, 128, 3, 72, "bf16"),     # exactly four key tiles, ragged token tail, odd head count
    (W.CROSS, 1, 31, 33, 16, 72, "bf16"),      # fewer tokens than one tile, one key past a tile edge
    (W.CROSS, 7, 333, 97, 8, 72, "bf16"),      # many tiles per wavefront, heads spread over the XCDs
    (W.CROSS, 3, 200, 60, 2, 32, "bf16"),
    (W.CROSS, 2, 150, 129, 2, 72, "bf16"),     # one key too many for the single-pass kernel: online softmax, K/V in LDS
    (W.CROSS, 17, 90, 300, 16, 72, "bf16"),    # config 4's text length: ten key tiles, the last ragged
    (W.CROSS, 3, 77, 192, 3, 72, "bf16"),      # fills the 6-tile LDS variant exactly
    (W.CROSS, 2, 100, 193, 2, 72, "bf16"),     # first length of the 8-tile variant
    (W.CROSS, 2, 61, 257, 5, 32, "bf16"),      # 10-tile variant, head dim 32
    (W.CROSS, 1, 45, 320, 2, 72, "bf16"),      # fills the 10-tile variant
    (W.CROSS, 2, 150, 321, 2, 72, "bf16"),     # 16-tile variant, 11 tiles in use
    (W.CROSS, 1, 40, 512, 2, 72, "bf16"),      # longest text the LDS-resident kernel takes
    (W.CROSS, 1, 40, 513, 2, 72, "bf16"),      # beyond it: streaming tile kernel
    (W.CROSS, 2, 64, 200, 2, 72, "f32"),       # fp32 rows: streaming tile kernel
]


@pytest.mark.parametrize("kind,T,S,L,H,D,dtype", SHAPES)
def test_attention_matches_oracle(pab, kind, T, S, L, H, D, dtype):
    print("case", W.KIND_NAMES[kind], T, S, L, H, D, dtype, flush=True)
    q, k, v = rand_qkv(kind, T, S, L, H, D, dtype, seed=1000 + 7 * T + S + L)
    out = pab.pab_attention_compute(kind, q.to(DEV), k.to(DEV), v.to(DEV))
    torch.cuda.synchronize()
    want = orc.kind_attention(kind, q, k, v)
    assert out.dtype == q.dtype and out.shape == q.shape
    assert_close(out, want, v, "shape case")
    if kind == W.TEMPORAL and T == 1:
        assert torch.equal(out.cpu(), v)
    if kind == W.CROSS and L == 1:
        assert torch.equal(out.cpu(), v.expand(T * S, H, D).reshape(T, S, H, D))


def test_peaked_queries_small(pab):
    # the stress configuration's value recipe (5% of query rows scaled by 8) at a size the
    # oracle can do in full: sharp and diffuse rows share tiles
    for kind, (T, S, L) in ((W.SPATIAL, (2, 333, 0)), (W.TEMPORAL, (16, 41, 0)), (W.CROSS, (2, 200, 120)),
                            (W.CROSS, (2, 200, 300))):
        q, k, v = rand_qkv(kind, T, S, L, 4, 72, "bf16", seed=77, scale_rows=0.05)
        out = pab.pab_attention_compute(kind, q.to(DEV), k.to(DEV), v.to(DEV))
        torch.cuda.synchronize()
        assert_close(out, orc.kind_attention(kind, q, k, v), v, "peaked %d" % kind)


def test_launches_follow_the_callers_stream(pab):
    # Two side streams (default priority) work on different inputs at once; each result is read after
    # synchronising only its own stream, and the scheduled call on a side stream leaves its slot filled.
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    cases = [(W.SPATIAL, 2, 300, 0), (W.TEMPORAL, 16, 50, 0), (W.CROSS, 2, 150, 120)]
    data = [rand_qkv(kind, T, S, L, 2, 72, "bf16", seed=300 + i) for i, (kind, T, S, L) in enumerate(cases)]
    dev = [tuple(x.to(DEV) for x in d) for d in data]
    torch.cuda.synchronize()
    outs = []
    for i, ((kind, T, S, L), (q, k, v)) in enumerate(zip(cases, dev)):
        st = (s1, s2)[i % 2]
        out = torch.full_like(q, float("nan"))
        st.wait_stream(torch.cuda.current_stream())     # the fill above ran on the current stream
        pab.pab_attention_compute(kind, q, k, v, out=out, stream=st)
        outs.append((st, out))
    for (st, out), (kind, T, S, L), (q, k, v) in zip(outs, cases, data):
        st.synchronize()
        assert_close(out, orc.kind_attention(kind, q, k, v), v, "side stream %d" % kind)
    wl = W.TINY
    ctx = pab.PabContext(pab.config_of(wl), DEV)
    q, k, v = W.make_qkv(wl, 0, W.SPATIAL, 0)
    with torch.cuda.stream(s1):
        dec, _ = ctx.pab_attention(0, W.SPATIAL, 0, q.to(DEV), k.to(DEV), v.to(DEV))
    s1.synchronize()
    assert dec == pab.COMPUTE
    assert_close(ctx.slot_tensor(0, W.SPATIAL), orc.kind_attention(W.SPATIAL, q, k, v), v, "scheduled call on a side stream")
    ctx.pab_destroy()


def test_compute_calls_replay_from_a_graph(pab):
    # The library neither allocates nor synchronises, so a run of launches can be captured once and replayed
    # (what a launch-bound loop such as the Tiny video wants).  Only this library's kernels are recorded; the
    # inputs are refreshed by eager copies between the replays and every replay is checked.
    cases = [(W.SPATIAL, 2, 300, 0), (W.TEMPORAL, 16, 50, 0), (W.CROSS, 2, 150, 120), (W.CROSS, 2, 150, 200)]
    shapes = [rand_qkv(kind, T, S, L, 2, 72, "bf16", seed=1) for kind, T, S, L in cases]
    static_in = [tuple(torch.empty_like(x, device=DEV) for x in d) for d in shapes]
    static_out = [torch.empty_like(d[0], device=DEV) for d in shapes]
    for (kind, T, S, L), (q, k, v), out in zip(cases, static_in, static_out):   # warm-up outside the capture
        q.zero_(); k.zero_(); v.zero_()
        pab.pab_attention_compute(kind, q, k, v, out=out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for (kind, T, S, L), (q, k, v), out in zip(cases, static_in, static_out):
            pab.pab_attention_compute(kind, q, k, v, out=out)
    for rep in range(3):
        data = [rand_qkv(kind, T, S, L, 2, 72, "bf16", seed=400 + 10 * rep + i) for i, (kind, T, S, L) in enumerate(cases)]
        for dst, src in zip(static_in, data):
            for a, b in zip(dst, src):
                a.copy_(b)
        for out in static_out:
            out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (kind, T, S, L), (q, k, v), out in zip(cases, data, static_out):
            assert_close(out, orc.kind_attention(kind, q, k, v), v, "replay %d kind %d" % (rep, kind))


def test_identical_keys_give_mean_of_values(pab):
    T, S, H, D = 1, 200, 2, 72
    q, k, v = rand_qkv(W.SPATIAL, T, S, 0, H, D, "bf16", seed=5)
    k = k[:, :1].expand(T, S, H, D).contiguous()
    out = pab.pab_attention_compute(W.SPATIAL, q.to(DEV), k.to(DEV), v.to(DEV)).cpu().double()
    mean = v.double().mean(1, keepdim=True).expand_as(out)
    assert (out - mean).abs().max() <= TOL * float(v.abs().max())


def test_tiny_video_every_cell(pab):
    """Config 1 end to end: every (step, block, kind) cell against the oracle's video run;
    reuse steps get NaN-poisoned q/k/v, must launch nothing and return the very bytes of
    the last computed step."""
    wl = W.TINY
    ctx = pab.PabContext(pab.config_of(wl), DEV)
    ctx.workspace.fill_(0xFF)            # NaN pattern: a slot read before being written would show
    vo = orc.VideoOracle(wl.intervals, wl.lo, wl.hi)
    poison = torch.full((wl.T, wl.S, wl.heads, wl.head_dim), float("nan"), device=DEV)
    last_bytes = {}
    last_vmax = {}
    computes = 0
    for step in range(wl.n_steps):
        for block, kind in wl.calls_per_step():
            want_dec = orc.schedule(step, wl.lo, wl.hi, wl.intervals[kind])
            if want_dec == orc.COMPUTE:
                q, k, v = W.make_qkv(wl, block, kind, step)
                dq, dk, dv = q.to(DEV), k.to(DEV), v.to(DEV)
            else:
                dq = dk = dv = poison
            before = ctx.pab_launch_count()
            dec, ptr = ctx.pab_attention(block, kind, step, dq, dk, dv)
            torch.cuda.synchronize()
            assert dec == want_dec
            assert ptr == ctx.pab_slot_ptr(block, kind)
            got = ctx.slot_tensor(block, kind)
            _, want = vo.step(block, kind, step, lambda: W.make_qkv(wl, block, kind, step))
            if dec == orc.COMPUTE:
                computes += 1
                assert ctx.pab_launch_count() == before + 1
                assert_close(got, want, v, "tiny step %d block %d kind %d" % (step, block, kind))
                last_bytes[(block, kind)] = got.clone()
                last_vmax[(block, kind)] = v.abs().max().reshape(1)
            else:
                assert ctx.pab_launch_count() == before
                assert torch.equal(got.view(torch.int32), last_bytes[(block, kind)].view(torch.int32))
                assert_close(got, want, last_vmax[(block, kind)], "tiny reuse")
    assert computes == ctx.pab_launch_count() == vo.computes == 2 * (7 + 5 + 5)
    # step going backwards without a reset is a state error; after reset it is fine
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl, 0, W.SPATIAL, 0))
    with pytest.raises(pab.PabError) as e:
        ctx.pab_attention(0, W.SPATIAL, 0, q, k, v)
    assert e.value.status == pab.ESTATE
    ctx.pab_reset()
    assert ctx.pab_launch_count() == 0
    with pytest.raises(pab.PabError) as e:       # reuse step first after reset: nothing cached
        ctx.pab_attention(0, W.SPATIAL, 3, None, None, None)
    assert e.value.status == pab.ESTATE
    for step in (0, 1, 2):
        dec, _ = ctx.pab_attention(0, W.SPATIAL, step, q, k, v)
        assert dec == pab.COMPUTE
    dec, _ = ctx.pab_attention(0, W.SPATIAL, 3, None, None, None)   # window step 3 reuses step 2; NULL inputs are fine
    assert dec == pab.REUSE
    torch.cuda.synchronize()
    ctx.pab_destroy()


def test_no_broadcast_baseline_computes_every_step(pab):
    wl = W.TINY
    ctx = pab.PabContext(pab.config_of(wl, (1, 1, 1)), DEV)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl, 0, W.TEMPORAL, 0))
    for step in range(wl.n_steps):
        dec, _ = ctx.pab_attention(1, W.TEMPORAL, step, q, k, v)
        assert dec == pab.COMPUTE
    torch.cuda.synchronize()
    assert ctx.pab_launch_count() == wl.n_steps


def test_tensors_beyond_four_gigabytes(pab):
    """Maximum sizes: q, k, v, o of 2.2 G elements (4.4 GB each), so element offsets pass 2^31 and byte offsets
    2^32 inside every tensor.  Spatial (2400 frames), temporal (120 000 positions per frame, 276 MB between the
    frames of a problem) and cross attention over the same buffers; frames / positions / tokens at the start, on
    both sides of the 2^31-element mark and at the very end are compared with the oracle, the rest is checked to
    be written and finite.  Inputs: torch's seeded generator on the device (N(0,1) rounded to bf16)."""
    H, D = 16, 72
    n = 2400 * 800 * H * D
    assert n > 2 ** 31
    g = torch.Generator(device=DEV)
    g.manual_seed(0x50414277)
    flat = [torch.randn(n, generator=g, device=DEV, dtype=torch.bfloat16) for _ in range(3)]
    out = torch.empty(n, device=DEV, dtype=torch.bfloat16)
    text_k, text_v = (torch.randn((120, H, D), generator=g, device=DEV, dtype=torch.bfloat16) for _ in range(2))

    def check(kind, T, S, picks):
        print("big", W.KIND_NAMES[kind], T, S, flush=True)
        q, k, v = (t.view(T, S, H, D) for t in flat)
        o = out.view(T, S, H, D)
        out.view(torch.int16).fill_(-1)                 # bf16 NaN pattern
        if kind == W.CROSS:
            pab.pab_attention_compute(kind, q, text_k, text_v, out=o)
        else:
            pab.pab_attention_compute(kind, q, k, v, out=o)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()), "unwritten or non-finite output"
        for pick in picks:
            if kind == W.SPATIAL:      # one frame is one batch entry
                sl = (slice(pick, pick + 1),)
            elif kind == W.TEMPORAL:   # one position is one batch entry
                sl = (slice(None), slice(pick, pick + 1))
            else:                      # eight tokens of frame pick
                sl = (slice(pick, pick + 1), slice(S - 8, S))
            qs, ks, vs = (t[sl].cpu() for t in (q, k, v))
            if kind == W.CROSS:
                ks, vs = text_k.cpu(), text_v.cpu()
            want = orc.kind_attention(kind, qs, ks, vs)
            assert_close(o[sl], want, vs, "big %s at %d" % (W.KIND_NAMES[kind], pick))

    mark = 2 ** 31 // (800 * H * D)                     # frame that holds element 2^31
    check(W.SPATIAL, 2400, 800, [0, mark - 1, mark, mark + 1, 2399])
    check(W.CROSS, 2400, 800, [0, mark, 2399])
    check(W.TEMPORAL, 16, 120000, [0, 59999, 119999])   # every problem spans 15 x 276 MB


def test_alternating_blocks_video(pab):
    """A Latte-shaped small video (config 3's structure: even blocks spatial only, odd blocks temporal only, no cross
    attention): with the per-block kind mask the slab holds one slot per block; every cell against the oracle's video
    run, and the cells that a block does not have are refused."""
    wl = W.Workload("alt_small", n_blocks=4, T=5, S=70, L=0, heads=3, head_dim=72, dtype="bf16", n_steps=8,
                    intervals=(2, 3, 0), lo=1, hi=6, alternating=True, seed=0x50414299)
    cfg = pab.config_of(wl)
    slot = (wl.T * wl.S * wl.heads * wl.head_dim * 2 + 255) // 256 * 256
    assert pab.pab_workspace_bytes(cfg) == 4 * slot
    ctx = pab.PabContext(cfg, DEV)
    ctx.workspace.fill_(0xFF)
    assert [ctx.pab_slot_ptr(b, k) for b in range(4) for k in range(3)] == \
        [ctx.workspace.data_ptr() + i * slot if k == i % 2 else 0 for i in range(4) for k in range(3)]
    vo = orc.VideoOracle(wl.intervals, wl.lo, wl.hi)
    last = {}
    for step in range(wl.n_steps):
        for block, kind in wl.calls_per_step():
            want_dec = orc.schedule(step, wl.lo, wl.hi, wl.intervals[kind])
            q = k = v = None
            if want_dec == orc.COMPUTE:
                q, k, v = W.make_qkv(wl, block, kind, step)
            dec, ptr = ctx.pab_attention(block, kind, step, *(t.to(DEV) if t is not None else None for t in (q, k, v)))
            torch.cuda.synchronize()
            assert dec == want_dec and ptr == ctx.workspace.data_ptr() + block * slot
            got = ctx.slot_tensor(block, kind)
            _, want = vo.step(block, kind, step, lambda: W.make_qkv(wl, block, kind, step))
            if dec == orc.COMPUTE:
                assert_close(got, want, v, "alternating step %d block %d kind %d" % (step, block, kind))
                last[block] = (got.clone(), v.abs().max().reshape(1))
            else:
                assert torch.equal(got.view(torch.int16), last[block][0].view(torch.int16))
                assert_close(got, want, last[block][1], "alternating reuse")
    assert ctx.pab_launch_count() == vo.computes
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl, 0, W.TEMPORAL, 0))
    with pytest.raises(pab.PabError) as e:       # block 0 is a spatial block
        ctx.pab_attention(0, W.TEMPORAL, 0, q, k, v)
    assert e.value.status == pab.EINVAL
    ctx.pab_destroy()


FULL = [(wl, kind) for wl in W.CONFIGS[1:] for kind in (W.SPATIAL, W.TEMPORAL, W.CROSS) if wl.intervals[kind] > 0]


@pytest.mark.parametrize("wl,kind", FULL, ids=lambda x: x.name if isinstance(x, W.Workload) else W.KIND_NAMES[x])
def test_full_size_every_row(pab, wl, kind):
    """Configs 2-5 at full size, in the launch configuration the benchmark times: one computed call per
    kind through the cache path into a slab poisoned with 0xFF, and EVERY output row compared with the
    oracle (a workgroup that wrote nothing, or wrote the wrong rows, cannot hide); then the reuse step."""
    print("full", wl.name, W.KIND_NAMES[kind], flush=True)
    small = W.Workload(wl.name, 1, wl.T, wl.S, wl.L, wl.heads, wl.head_dim, wl.dtype, wl.n_steps,
                       wl.intervals, wl.lo, wl.hi, peaked_frac=wl.peaked_frac, seed=wl.seed)
    ctx = pab.PabContext(pab.config_of(small), DEV)
    ctx.workspace.fill_(0xFF)         # bf16 0xFFFF is a NaN: anything left unwritten fails the comparison
    step = wl.lo                      # first step of the window: computed
    q, k, v = W.make_qkv(small, 0, kind, step)
    dq, dk, dv = q.to(DEV), k.to(DEV), v.to(DEV)
    dec, _ = ctx.pab_attention(0, kind, step, dq, dk, dv)
    assert dec == pab.COMPUTE
    torch.cuda.synchronize()
    out = ctx.slot_tensor(0, kind)
    want = orc.kind_attention(kind, q, k, v)
    err = assert_close(out, want, v, "%s %s, all rows" % (wl.name, W.KIND_NAMES[kind]))
    print("  max abs err %.3e = %.2f of the bound" % (err, err / (TOL * float(v.abs().max()))), flush=True)
    # the slots of the other kinds were not touched
    for other in (W.SPATIAL, W.TEMPORAL, W.CROSS):
        if other != kind and wl.intervals[other] > 0:
            assert bool((ctx.slot_tensor(0, other).view(torch.int16) == -1).all())
    # the next step of the window reuses: same pointer, same bytes, nothing launched
    snap = out.clone()
    dec, _ = ctx.pab_attention(0, kind, step + 1, None, None, None)
    if wl.intervals[kind] > 1:
        assert dec == pab.REUSE and ctx.pab_launch_count() == 1
        assert torch.equal(ctx.slot_tensor(0, kind).view(torch.int16), snap.view(torch.int16))
    ctx.pab_destroy()


def test_full_size_slab_addressing(pab):
    """Config 2's shape with 3 blocks x 3 kinds: nine computed calls with distinct inputs into a poisoned slab of
    nine 58.6 MB slots; each slot is compared with the oracle's output for ITS inputs (every row for temporal and
    cross, every row of four (frame, head) pairs plus 2000 seeded rows for spatial), so a call that landed in
    another cell's slot, or spilled over a slot boundary, shows."""
    wl = W.OPENSORA_480P
    three = W.Workload(wl.name, 3, wl.T, wl.S, wl.L, wl.heads, wl.head_dim, wl.dtype, wl.n_steps, wl.intervals, wl.lo,
                       wl.hi, seed=wl.seed)
    ctx = pab.PabContext(pab.config_of(three), DEV)
    ctx.workspace.fill_(0xFF)
    slot_bytes = wl.T * wl.S * wl.heads * wl.head_dim * 2
    assert ctx.workspace.numel() == 9 * slot_bytes
    cells = [(b, kind) for b in range(3) for kind in (W.SPATIAL, W.TEMPORAL, W.CROSS)]
    order = [cells[i] for i in (4, 0, 8, 2, 6, 1, 5, 3, 7)]     # not in slab order
    inputs = {}
    for n, (b, kind) in enumerate(order):
        print("slab cell", b, W.KIND_NAMES[kind], flush=True)
        q, k, v = W.make_qkv(three, b, kind, 0)
        inputs[(b, kind)] = (q, k, v)
        dec, ptr = ctx.pab_attention(b, kind, 0, q.to(DEV), k.to(DEV), v.to(DEV))
        assert dec == pab.COMPUTE
        assert ptr == ctx.workspace.data_ptr() + (3 * b + kind) * slot_bytes
        torch.cuda.synchronize()
        # the cells not yet computed are still poison, bit for bit
        for (b2, k2) in order[n + 1:]:
            assert bool((ctx.slot_tensor(b2, k2).view(torch.int16) == -1).all()), (b, kind, b2, k2)
    assert ctx.pab_launch_count() == 9
    for (b, kind) in cells:
        q, k, v = inputs[(b, kind)]
        got = ctx.slot_tensor(b, kind).cpu()
        assert bool(torch.isfinite(got).all()), (b, kind)
        if kind == W.SPATIAL:
            for t, h in ((0, 0), (wl.T - 1, wl.heads - 1), (5, 3 + b), (9 + b, 12)):
                want = orc.spatial(q[t:t + 1, :, h:h + 1], k[t:t + 1, :, h:h + 1], v[t:t + 1, :, h:h + 1])
                assert_close(got[t:t + 1, :, h:h + 1], want, v, "slab spatial block %d frame %d head %d" % (b, t, h))
            rows = W.sample_rows(three, 2000, seed=100 + b)
            want = orc.attention_rows(kind, q, k, v, rows)
            err = np.abs(got[rows[:, 0], rows[:, 1], rows[:, 2]].double().numpy() - want).max()
            assert err <= TOL * float(v.abs().max()), (b, err)
        else:
            assert_close(got, orc.kind_attention(kind, q, k, v), v, "slab block %d kind %d" % (b, kind))
    ctx.pab_destroy()


def test_reuse_refuses_a_slot_that_holds_another_step(pab):
    """Eq. 1 broadcasts from one particular computed step.  A caller that skipped that step for a cell (here the
    window opens at step 3 with range 4, and the cell is called at steps 0, 1, 2 and then 4) must get PAB_ESTATE
    at the reuse step, not the stale output of step 2."""
    wl = W.Workload("skip", 1, 4, 64, 16, 4, 32, "f32", 10, (4, 4, 4), 3, 8, seed=5)
    ctx = pab.PabContext(pab.config_of(wl), DEV)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl, 0, W.SPATIAL, 0))
    for step in (0, 1, 2):
        assert ctx.pab_attention(0, W.SPATIAL, step, q, k, v)[0] == pab.COMPUTE
    with pytest.raises(pab.PabError) as e:
        ctx.pab_attention(0, W.SPATIAL, 4, None, None, None)
    assert e.value.status == pab.ESTATE and "needs the output of step 3" in str(e.value)
    # the same cell played without the gap is fine
    ctx.pab_reset()
    for step in (0, 1, 2, 3):
        assert ctx.pab_attention(0, W.SPATIAL, step, q, k, v)[0] == pab.COMPUTE
    assert ctx.pab_attention(0, W.SPATIAL, 4, None, None, None)[0] == pab.REUSE
    torch.cuda.synchronize()
    ctx.pab_destroy()


def test_video_with_window_from_preset_and_timesteps(pab):
    """App. A.2.1 end to end: the broadcast ranges and the timestep window come from pab_preset, the window is
    mapped onto a synthetic sampler's timestep list by pab_window_from_timesteps, and a small video is played
    through pab_attention with that configuration, every cell against the oracle's video run (which maps the
    same window with the oracle's own routine)."""
    n_steps = 12
    timesteps = [1000.0 - 1000.0 * s / n_steps for s in range(n_steps)]      # 1000, 916.7, ..., 83.3
    for model, level in ((0, 0), (2, 1)):
        intervals, t_start, t_end = pab.pab_preset(model, level)
        lo, hi = pab.pab_window_from_timesteps(timesteps, t_start, t_end)
        assert (lo, hi) == orc.window_from_timesteps(timesteps, t_start, t_end)
        assert 0 < lo < hi < n_steps - 1
        wl = W.Workload("preset_%d_%d" % (model, level), 2, 3, 50, 24, 2, 72, "bf16", n_steps, tuple(intervals), lo, hi,
                        seed=40 + model)
        ctx = pab.PabContext(pab.config_of(wl), DEV)
        ctx.workspace.fill_(0xFF)
        vo = orc.VideoOracle(wl.intervals, lo, hi)
        last = {}
        for step in range(n_steps):
            for block, kind in wl.calls_per_step():
                want_dec, want = vo.step(block, kind, step, lambda: W.make_qkv(wl, block, kind, step))
                if want_dec == orc.COMPUTE:
                    q, k, v = W.make_qkv(wl, block, kind, step)
                    dec, _ = ctx.pab_attention(block, kind, step, q.to(DEV), k.to(DEV), v.to(DEV))
                    last[(block, kind)] = v.abs().max().reshape(1)
                else:
                    dec, _ = ctx.pab_attention(block, kind, step, None, None, None)
                torch.cuda.synchronize()
                assert dec == want_dec, (model, step, block, kind)
                assert_close(ctx.slot_tensor(block, kind), want, last[(block, kind)], "preset video step %d" % step)
        assert ctx.pab_launch_count() == vo.computes
        ctx.pab_destroy()


def test_long_spatial_and_long_text_shapes(pab):
    """Seeded shapes where the steady loops of the tiled kernels run many times: spatial attention with up to
    2600 tokens (both dtypes, both head dims, 5% of the query rows scaled x8 in some of the bf16 cases), and cross
    attention over 129..512 text tokens, each compared in full with the oracle."""
    rng = np.random.default_rng(20241128)
    worst = 0.0
    cases = []
    for i in range(14):
        cases.append((W.SPATIAL, 1, int(rng.integers(257, 2601)), 0, int(rng.integers(1, 3)), int(rng.choice([72, 72, 32])),
                      "bf16" if i % 3 else "f32", 0.05 if i % 2 and i % 3 else 0.0))
    for L in (129, 191, 192, 193, 255, 256, 257, 319, 320, 321, 400, 511, 512):
        cases.append((W.CROSS, 1, int(rng.integers(33, 400)), L, int(rng.integers(1, 5)), 72, "bf16", 0.05 if L % 2 else 0.0))
    for n, (kind, T, S, L, H, D, dtype, peaked) in enumerate(cases):
        print("long case", n, W.KIND_NAMES[kind], T, S, L, H, D, dtype, peaked, flush=True)
        q, k, v = rand_qkv(kind, T, S, L, H, D, dtype, seed=7000 + n, scale_rows=peaked)
        out = pab.pab_attention_compute(kind, q.to(DEV), k.to(DEV), v.to(DEV))
        torch.cuda.synchronize()
        err = assert_close(out, orc.kind_attention(kind, q, k, v), v, "long case %d" % n)
        worst = max(worst, err / (TOL * float(v.abs().max())))
    print("worst error / bound over the long cases: %.2f" % worst)


def test_seeded_random_shapes(pab):
    """Sixty seeded shapes across kinds, dtypes, head dims and all kernel variants (tile, temporal 16/24/32-row and
    tiled fallback, cross single-pass / LDS-resident online / tiled), each compared in full with the oracle."""
    rng = np.random.default_rng(20241127)
    worst = 0.0
    for case in range(60):
        kind = int(rng.integers(0, 3))
        D = int(rng.choice([32, 72]))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        H = int(rng.integers(1, 9))
        if kind == W.SPATIAL:
            T, S, L = int(rng.integers(1, 4)), int(rng.integers(1, 420)), 0
        elif kind == W.TEMPORAL:
            T, S, L = int(rng.integers(1, 41)), int(rng.integers(1, 60)), 0
        else:
            T, S, L = int(rng.integers(1, 4)), int(rng.integers(1, 200)), int(rng.choice([1, 7, 31, 32, 33, 100, 128, 129, 191, 256, 300, 511, 512, 530]))
        print("fuzz case", case, W.KIND_NAMES[kind], T, S, L, H, D, dtype, flush=True)
        q, k, v = rand_qkv(kind, T, S, L, H, D, dtype, seed=5000 + case)
        out = pab.pab_attention_compute(kind, q.to(DEV), k.to(DEV), v.to(DEV))
        torch.cuda.synchronize()
        err = assert_close(out, orc.kind_attention(kind, q, k, v), v, "fuzz case %d" % case)
        worst = max(worst, err / (TOL * float(v.abs().max())))
    print("worst error / bound over the fuzz cases: %.2f" % worst)
