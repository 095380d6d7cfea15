"""GPU parity: the HIP library against the fp64 oracle, element by element, through the C ABI.

Inputs are seeded and synthetic (paper_2409_09086_amd.workloads); the oracle runs on the host in
the same process.  Bars: attention output max-abs 2e-2 (bf16) / 1e-4 (fp32); retained sets
identical up to keys within 1e-5 relative of the r-th largest fp64 score.
"""
import numpy as np
import pytest
import torch

from oracle import OracleStream
from paper_2409_09086_amd import binding as B
from paper_2409_09086_amd.workloads import CONFIGS, ChunkStream, random_chunk
from _parity import LockStep, OUT_TOL

pytestmark = pytest.mark.gpu
DT = {"fp32": torch.float32, "bf16": torch.bfloat16}


def pair(budget, recent, heads, kv, d, dtype, bias, max_chunk=None, impl=None, scale=None, max_decode=None,
         attn_tile=None):
    gpu = B.Stream(budget, recent, heads, kv, d, dtype=DT[dtype], bias=bias, max_chunk=max_chunk, impl=impl, scale=scale,
                   max_decode=max_decode, attn_tile=attn_tile)
    # the oracle is given b and the scale as the doubles the library is given (default scale: 1/sqrt(d))
    orc = OracleStream(budget, recent, heads, kv, d, bias=bias, scale=scale)
    return LockStep(gpu, orc)


@pytest.mark.parametrize("bias", [0.0, 1e-4, 1e-2, 1.0, 512.0])
def test_cfg1_tiny_fp32_stream(bias):
    cfg = CONFIGS["cfg1"]
    ls = pair(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.dtype, bias, max_chunk=cfg.max_chunk)
    for step, (q, k, v) in zip(range(cfg.steps), ChunkStream(cfg)):
        print("cfg1 bias", bias, "step", step, flush=True)
        ls.step(q, k, v, check_state=True)
    assert len(ls.gpu) == cfg.budget and ls.gpu.streamed == cfg.steps * cfg.chunk
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


@pytest.mark.parametrize("impl", [1, 0])
@pytest.mark.parametrize("heads,kv,d,budget,recent,chunks", [
    (4, 4, 128, 192, 64, [64, 64, 64, 64, 64, 64]),
    (8, 2, 128, 160, 48, [100, 37, 64, 1, 129, 77, 5, 160]),      # GQA, ragged, L=1, L up to budget
    (4, 2, 64, 96, 96, [32, 64, 50, 50]),                           # r = 0: pure window
    (2, 2, 64, 128, 0, [64, 64, 64, 64]),                           # R = 0: nothing pinned
    (4, 1, 128, 200, 150, [70, 70, 70, 70, 70]),                    # R > L
    (6, 2, 128, 128, 40, [60, 60, 33, 60, 60]),                     # group of 3 query heads
    (8, 1, 64, 96, 32, [48, 48, 48, 48]),                           # group of 8 query heads
    (2, 2, 128, 300, 100, [300, 7, 300, 150]),                      # chunk as long as the budget
    (4, 2, 128, 96, 32, [150, 40, 150, 1, 97]),                     # chunks longer than the budget: the first step evicts
    (2, 2, 64, 24, 8, [40, 3, 17, 24, 5]),                          # budget below one 32-row tile
    (2, 1, 128, 40, 40, [64, 9]),                                   # r = 0 and chunk > budget
    (8, 2, 128, 256, 128, [128, 128, 128, 128]),                    # scored rows shared out over 2 workgroups
    (4, 1, 128, 384, 192, [192, 192, 192, 101, 192]),               # ... over 3
    (16, 2, 64, 320, 160, [160, 160, 160, 45, 160]),                # ... over 4, uneven shares, ragged last block
    (32, 32, 128, 640, 128, [576, 608, 576, 530]),                  # full head count, chunks of 9 and 10 row tiles
])
def test_small_bf16_streams(impl, heads, kv, d, budget, recent, chunks):
    ls = pair(budget, recent, heads, kv, d, "bf16", 1e-3, max_chunk=max(chunks), impl=impl)
    for step, L in enumerate(chunks):
        print("bf16 impl", impl, (heads, kv, d, budget, recent), "step", step, "L", L, flush=True)
        q, k, v = random_chunk(100 + step, L, heads, kv, d, "bf16")
        ls.step(q, k, v, check_state=True)
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


def test_import_then_step_matches_oracle():
    heads, kv, d, budget, recent, L = 4, 2, 128, 128, 32, 48
    ls = pair(budget, recent, heads, kv, d, "bf16", 1e-2, max_chunk=L, impl=1)
    g = torch.Generator().manual_seed(7)
    K = torch.randn((kv, budget, d), generator=g).bfloat16()
    V = torch.randn((kv, budget, d), generator=g).bfloat16()
    pos = torch.arange(0, 3 * budget, 3, dtype=torch.int32).repeat(kv, 1)
    ls.gpu.load(K.cuda(), V.cuda(), pos.cuda().contiguous(), 5000)
    ls.oracle.load(K.double().numpy(), V.double().numpy(), pos.numpy(), 5000)
    q, k, v = random_chunk(8, L, heads, kv, d, "bf16")
    ls.step(q, k, v, check_state=True)
    assert ls.gpu.streamed == 5000 + L
    _, _, p, score = ls.gpu.export()
    score = score.cpu().numpy()
    assert np.isinf(score[:, budget - recent:]).all() and np.isfinite(score[:, : budget - recent]).all()


def test_step_errors_leave_the_stream_unchanged():
    s = B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, max_chunk=32, impl=1)
    q, k, v = [x.cuda() for x in random_chunk(1, 33, 2, 2, 64, "bf16")]
    with pytest.raises(B.InfMLLMError) as e:
        s.step(q, k, v)
    assert e.value.code == B.ECAPACITY and len(s) == 0 and s.streamed == 0


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("heads,kv,budget,recent,chunks", [
    (4, 4, 192, 64, [64, 100, 37, 129, 192, 1, 77]),                # ragged chunks, causal tiles of every shape
    (8, 2, 320, 128, [128, 128, 128, 45, 128]),                     # grouped heads: row blocks of one tile span heads
])
def test_every_attention_tile_shape(tile, heads, kv, budget, recent, chunks):
    """INFMLLM_PARAM_ATTN_TILE forces each workgroup shape of the matrix-core attention (head_dim 128) in turn;
    the launch normally picks one from the chunk length, so small streams would only ever reach one of them."""
    ls = pair(budget, recent, heads, kv, 128, "bf16", 1e-3, max_chunk=max(chunks), attn_tile=tile)
    for step, L in enumerate(chunks):
        print("tile", tile, (heads, kv, budget, recent), "step", step, "L", L, flush=True)
        q, k, v = random_chunk(1200 + step, L, heads, kv, 128, "bf16")
        ls.step(q, k, v, check_state=True)
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


@pytest.mark.parametrize("heads,kv,budget,recent,chunks", [
    (4, 4, 768, 256, [768, 512, 300]),          # one head per wavefront: four pairs of row blocks per workgroup
    (8, 2, 512, 192, [512, 448]),               # groups of four heads share a workgroup's K/V tiles
    (4, 2, 512, 128, [512, 512, 200]),          # groups of two
])
def test_attention_row_block_pairs_on_long_chunks(heads, kv, budget, recent, chunks):
    """The 64-rows-per-wavefront attention pairs a row block from the front of the chunk with one from its back
    and finishes the back one alone.  Chunks of several hundred rows make every phase of that loop last several
    tiles (both blocks, both blocks with block A masked, block B alone, block B masked), with ragged chunk
    lengths leaving some back blocks empty; every output element is compared with the oracle."""
    ls = pair(budget, recent, heads, kv, 128, "bf16", 1e-3, max_chunk=max(chunks), attn_tile=5)
    for step, L in enumerate(chunks):
        print("pairs", (heads, kv, budget, recent), "step", step, "L", L, flush=True)
        q, k, v = random_chunk(1300 + step, L, heads, kv, 128, "bf16")
        ls.step(q, k, v, check_state=True)
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


def test_bad_attention_tile_is_refused():
    with pytest.raises(B.InfMLLMError) as e:
        B.Stream(64, 16, 2, 2, 128, dtype=torch.bfloat16, attn_tile=6)
    assert e.value.code == B.EINVAL


@pytest.mark.parametrize("name,steps", [("cfg2", 64), ("cfg3", 17), ("cfg4", 13), ("cfg5", 6)])
def test_full_shape_streams_lockstep(name, steps):
    """The real layer shapes in the launch configuration the benchmark times, every output element and every
    retained set against the oracle: cfg2 for its whole stream of 64 chunks, cfg3 for 4 warm-up and 13 evicting
    steps, cfg4 and cfg5 for their warm-up and first evicting steps (their later steps: the spot checks below)."""
    cfg = CONFIGS[name]
    ls = pair(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.dtype, cfg.bias, max_chunk=cfg.max_chunk)
    for step, (q, k, v) in zip(range(steps), ChunkStream(cfg)):
        print(name, "step", step, flush=True)
        ls.step(q, k, v, check_state=(step == steps - 1))
    print("%s: max err %.3g swaps %d" % (name, ls.max_err, ls.swaps), flush=True)


@pytest.mark.parametrize("name,steps", [("cfg2", 30), ("cfg3", 12), ("cfg4", 30), ("cfg5", 12)])
def test_step_properties_at_the_real_shapes(name, steps):
    """A property that holds at any size, checked at the real shapes over many steps without the oracle: the
    list a step reports is exactly Alg. 1 l.5-7 applied to the scores W' the library itself reports for that
    step (r largest, ties to the newer row, ascending, then the recent window), and the cache after the step is
    the cache before it followed by the chunk, gathered by that list (Alg. 1 l.8), bit for bit.  This isolates
    the selection kernel (two, four and eight candidates per thread at these shapes) and the gather from the
    precision of the scores.  Every fourth step the chunk's output is also compared with torch's fp32 arithmetic
    on the same cache and chunk (2e-2)."""
    cfg = CONFIGS[name]
    gpu = B.Stream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, dtype=DT[cfg.dtype], bias=cfg.bias,
                   max_chunk=cfg.max_chunk)
    r = cfg.budget - cfg.recent
    checked = 0
    for step, (q, k, v) in zip(range(steps), ChunkStream(cfg)):
        t, T = len(gpu), gpu.streamed
        n = t + q.shape[0]
        K0, V0, pos0, _ = gpu.export()
        out_g, ret, cnt = gpu.step(q.cuda(), k.cuda(), v.cuda())
        if n <= cfg.budget:
            continue
        w = gpu.last_scores().cpu().numpy()                           # [kv_heads, c], fp32 as ranked
        I = ret.cpu().numpy()[:, : int(cnt.item())]
        c = n - cfg.recent
        assert w.shape == (cfg.kv_heads, c)
        for h in range(cfg.kv_heads):
            order = np.lexsort((-np.arange(c), -w[h].astype(np.float64)))   # by score descending, then newer first
            assert (I[h, :r] == np.sort(order[:r])).all(), (name, step, h)
            assert (I[h, r:] == np.arange(c, n)).all()
        # Alg. 1 l.8: the new cache is the old cache followed by the chunk, gathered by that list, bit for bit
        K1, V1, pos1, _ = gpu.export()
        if step % 4 == 0:
            # Sec. 3.2: the chunk's output against torch's own fp32 arithmetic on the same cache and chunk
            G = cfg.heads // cfg.kv_heads
            Kf = torch.cat([K0, k.cuda().permute(1, 0, 2)], dim=1).float().repeat_interleave(G, dim=0)   # [Hq, n, d]
            Vf = torch.cat([V0, v.cuda().permute(1, 0, 2)], dim=1).float().repeat_interleave(G, dim=0)
            s_ = torch.einsum("lhd,hnd->hln", q.cuda().float(), Kf) / np.sqrt(cfg.head_dim)
            L_ = q.shape[0]
            vis = torch.arange(n, device="cuda")[None, :] <= (t + torch.arange(L_, device="cuda"))[:, None]
            ref = torch.einsum("hln,hnd->lhd", torch.softmax(s_.masked_fill(~vis[None], float("-inf")), dim=-1), Vf)
            err = float((out_g.float() - ref).abs().max())
            assert err <= 2e-2, (name, step, err)
        Kall = torch.cat([K0, k.cuda().permute(1, 0, 2)], dim=1)
        Vall = torch.cat([V0, v.cuda().permute(1, 0, 2)], dim=1)
        pall = torch.cat([pos0, torch.arange(T, T + q.shape[0], dtype=torch.int32, device="cuda").repeat(cfg.kv_heads, 1)], dim=1)
        idx = ret[:, : int(cnt.item())].long()
        assert torch.equal(K1, torch.gather(Kall, 1, idx[:, :, None].expand(-1, -1, cfg.head_dim)))
        assert torch.equal(V1, torch.gather(Vall, 1, idx[:, :, None].expand(-1, -1, cfg.head_dim)))
        assert torch.equal(pos1, torch.gather(pall, 1, idx))
        checked += 1
    assert checked >= steps // 2
    print("%s: %d evicting steps checked" % (name, checked), flush=True)


@pytest.mark.parametrize("name,skip,steps,layer", [("cfg2", 40, 3, 0), ("cfg3", 60, 3, 0), ("cfg4", 25, 5, 0),
                                                   ("cfg4", 37, 4, 1), ("cfg5", 47, 3, 0), ("cfg5", 96, 3, 1)])
def test_late_steps_spot_check(name, skip, steps, layer):
    """Steps far into a stream, which the oracle cannot reach on its own: the GPU runs `skip`
    steps alone, the oracle adopts the exported cache (bit-exact rows and positions), and the
    next steps are compared in lock-step.  cfg5's windows cover the chunks at 100 000 tokens (layer 0) and at
    200 000 tokens (layer 1's own sub-seeded stream) in which the recurring key bank returns, and the step after
    each; cfg4's cover frames with a trailing text query (steps 29 and 39), the second on layer 1's stream."""
    cfg = CONFIGS[name]
    ls = pair(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.dtype, cfg.bias, max_chunk=cfg.max_chunk)
    stream = ChunkStream(cfg, layer=layer)
    for step in range(skip):
        ls.gpu_only(*next(stream))
        if step % 16 == 15:
            print(name, "layer", layer, "unchecked step", step, flush=True)
    torch.cuda.synchronize()
    assert len(ls.gpu) == cfg.budget
    pos = ls.gpu.positions().cpu().numpy()
    assert (np.diff(pos, axis=1) > 0).all() and pos.max() < ls.gpu.streamed
    assert (pos[:, -cfg.recent:] == np.arange(ls.gpu.streamed - cfg.recent, ls.gpu.streamed)).all()
    ls.adopt_gpu_state()
    for step in range(skip, skip + steps):
        print(name, "late step", step, flush=True)
        ls.step(*next(stream), check_state=(step == skip + steps - 1))
    print("%s layer %d late: max err %.3g swaps %d" % (name, layer, ls.max_err, ls.swaps), flush=True)


def test_more_candidates_than_fit_in_registers():
    """c > 16384 candidates per head takes the selection kernel that keeps the scores in memory."""
    heads, kv, d, budget, recent, L = 2, 1, 64, 17000, 200, 128
    ls = pair(budget, recent, heads, kv, d, "bf16", 1e-3, max_chunk=budget)
    g = torch.Generator().manual_seed(11)
    K = torch.randn((kv, budget, d), generator=g).bfloat16()
    V = torch.randn((kv, budget, d), generator=g).bfloat16()
    pos = torch.arange(budget, dtype=torch.int32).repeat(kv, 1)
    ls.gpu.load(K.cuda(), V.cuda(), pos.cuda().contiguous(), budget)
    ls.oracle.load(K.double().numpy(), V.double().numpy(), pos.numpy(), budget)
    for step in range(2):
        q, k, v = random_chunk(20 + step, L, heads, kv, d, "bf16")
        ls.step(q, k, v, check_state=True)
    assert ls.gpu.last_scores().shape == (kv, budget + L - recent)


def test_sixteen_candidates_per_thread():
    """8192 < c <= 16384 candidates per head: the selection keeps sixteen keys per thread in registers."""
    heads, kv, d, budget, recent, L = 2, 1, 64, 12100, 200, 128
    ls = pair(budget, recent, heads, kv, d, "bf16", 1e-3, max_chunk=L)
    g = torch.Generator().manual_seed(12)
    K = torch.randn((kv, budget, d), generator=g).bfloat16()
    V = torch.randn((kv, budget, d), generator=g).bfloat16()
    pos = torch.arange(budget, dtype=torch.int32).repeat(kv, 1)
    ls.gpu.load(K.cuda(), V.cuda(), pos.cuda().contiguous(), budget)
    ls.oracle.load(K.double().numpy(), V.double().numpy(), pos.numpy(), budget)
    for step in range(2):
        q, k, v = random_chunk(30 + step, L, heads, kv, d, "bf16")
        ls.step(q, k, v, check_state=True)
    assert ls.gpu.last_scores().shape == (kv, budget + L - recent)


@pytest.mark.parametrize("d", [128, 64])
def test_more_scored_rows_than_the_scoring_kernel_keeps_in_lds(d):
    """G * l_q = 8 * 1024 scored rows per kv-head: beyond 4096 the scoring kernel reads each staged row's
    log-sum-exp from memory instead of from its LDS copy."""
    heads, kv, budget, recent, L = 8, 1, 2048, 1024, 1024
    ls = pair(budget, recent, heads, kv, d, "bf16", 1e-3, max_chunk=L)
    for step in range(4):                                          # two warm-up steps, two evicting ones
        print("direct lse d", d, "step", step, flush=True)
        q, k, v = random_chunk(1300 + step, L, heads, kv, d, "bf16")
        ls.step(q, k, v, check_state=(step == 3))
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


@pytest.mark.parametrize("d", [64, 128])
def test_fp32_streams_with_grouped_heads(d):
    ls = pair(160, 48, 8, 2, d, "fp32", 1e-2, max_chunk=100)
    for step, L in enumerate([100, 37, 64, 1, 77]):
        q, k, v = random_chunk(300 + step, L, 8, 2, d, "fp32")
        ls.step(q, k, v, check_state=True)


def test_scores_reported_match_oracle_scores():
    """W' itself (not only its ranking) against the fp64 scores, through infmllm_stream_last_scores."""
    heads, kv, d, budget, recent, L = 8, 2, 128, 512, 128, 128
    ls = pair(budget, recent, heads, kv, d, "bf16", 1e-3, max_chunk=L)
    for step in range(6):
        q, k, v = random_chunk(400 + step, L, heads, kv, d, "bf16")
        dev = ls.gpu.device
        t = len(ls.oracle)
        ls.gpu.step(q.to(dev), k.to(dev), v.to(dev))
        ls.oracle.attend(q.double().numpy(), k.double().numpy(), v.double().numpy())
        sc = ls.oracle.scores()
        w = ls.gpu.last_scores()
        if sc is None:
            assert w is None
        else:
            S, Wb = sc
            err = np.abs(w.double().cpu().numpy() - Wb).max()
            assert err <= 2e-6 * np.abs(S).max() + 1e-9, err
        ls.oracle.commit(ls.oracle.select())
    # the two sides selected independently here; they must still agree on the final cache
    ls.check_state()


def test_scores_do_not_depend_on_workgroup_order():
    """Where the scored rows of a column block are shared out over several workgroups, whichever finishes last
    adds the slices up; the slices are added in slice order, so W' is the same bits on every run."""
    heads, kv, d, budget, recent, L = 16, 2, 64, 320, 160, 160          # four slices per column block
    chunks = [random_chunk(900 + step, L, heads, kv, d, "bf16") for step in range(4)]
    seen = None
    for rep in range(6):
        gpu = B.Stream(budget, recent, heads, kv, d, dtype=torch.bfloat16, bias=1e-3, max_chunk=L)
        ws = []
        for q, k, v in chunks:
            _, ret, _ = gpu.step(q.cuda(), k.cuda(), v.cuda())
            w = gpu.last_scores()
            ws.append(None if w is None else w.clone())
        torch.cuda.synchronize()
        assert ws[-1] is not None
        if seen is None:
            seen = ws
        else:
            for a, b in zip(seen, ws):
                assert (a is None) == (b is None)
                if a is not None:
                    assert torch.equal(a.view(torch.int32), b.view(torch.int32)), "scores differ between runs"


# ---------------------------------------------------------------------------------------
# decoding steps (Sec. 3.2: no eviction while tokens are decoded)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("heads,kv,d,dtype", [(4, 4, 128, "bf16"), (8, 2, 128, "bf16"), (8, 1, 64, "bf16"),
                                              (4, 2, 64, "fp32"), (6, 1, 128, "fp32")])
def test_decode_steps_between_chunks(heads, kv, d, dtype):
    budget, recent, L, nd = 192, 48, 64, 9
    ls = pair(budget, recent, heads, kv, d, dtype, 1e-3, max_chunk=L, max_decode=nd)
    key = 0
    for rnd in range(5):                                         # rounds of (prompt chunk, a few decoded tokens)
        q, k, v = random_chunk(500 + rnd, L, heads, kv, d, dtype)
        ls.step(q, k, v, check_state=True)
        for i in range(nd if rnd % 2 == 0 else 3):
            key += 1
            q1, k1, v1 = random_chunk(600 + key, 1, heads, kv, d, dtype)
            ls.decode(q1, k1, v1)
        ls.check_state()                                         # the cache may exceed the budget here
    assert len(ls.gpu) <= ls.gpu.max_len == budget + nd
    assert len(ls.gpu) == budget + nd                            # the last round decoded max_decode tokens
    q1, k1, v1 = [x.cuda() for x in random_chunk(1, 1, heads, kv, d, dtype)]
    with pytest.raises(B.InfMLLMError) as e:                     # budget + max_decode rows are cached
        ls.gpu.decode(q1, k1, v1)
    assert e.value.code == B.ECAPACITY


def test_decode_at_full_shape_cfg2():
    """cfg2's layer shape with the cache full: 16 decoded tokens, then the next prompt evicts."""
    cfg = CONFIGS["cfg2"]
    ls = pair(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.dtype, cfg.bias,
              max_chunk=cfg.max_chunk, max_decode=16)
    stream = ChunkStream(cfg)
    for step in range(5):
        ls.step(*next(stream))
    for i in range(16):
        q1, k1, v1 = random_chunk(700 + i, 1, cfg.heads, cfg.kv_heads, cfg.head_dim, "bf16", sigma=0.5)
        ls.decode(q1, k1, v1)
    assert len(ls.gpu) == cfg.budget + 16
    ls.step(*next(stream), check_state=True)
    assert len(ls.gpu) == cfg.budget
    print("decode cfg2: max err %.3g swaps %d" % (ls.max_err, ls.swaps), flush=True)


@pytest.mark.parametrize("heads,kv,d,dtype", [(8, 2, 128, "bf16"), (4, 2, 64, "fp32")])
def test_decode_n_equals_token_by_token(heads, kv, d, dtype):
    """infmllm_decode_n enqueues n decoding steps from one call: outputs against the oracle token by token, and the
    outputs and the cache bit for bit against a twin stream that calls infmllm_decode once per token."""
    budget, recent, L, nd = 192, 48, 64, 12
    ls = pair(budget, recent, heads, kv, d, dtype, 1e-3, max_chunk=L, max_decode=nd)
    twin = B.Stream(budget, recent, heads, kv, d, dtype=ls.gpu.dtype, bias=1e-3, max_chunk=L, max_decode=nd)
    for rnd in range(4):
        q, k, v = random_chunk(520 + rnd, L, heads, kv, d, dtype)
        ls.step(q, k, v, check_state=True)
        twin.step(q.cuda(), k.cuda(), v.cuda())
        n = (nd, 1, 5, nd)[rnd]
        qn, kn, vn = random_chunk(620 + rnd, n, heads, kv, d, dtype)
        out_n = ls.gpu.decode_n(qn.cuda(), kn.cuda(), vn.cuda())
        for i in range(n):
            out_o = ls.oracle.decode(qn[i:i + 1].double().numpy(), kn[i:i + 1].double().numpy(), vn[i:i + 1].double().numpy())
            err = float(np.abs(out_n[i:i + 1].double().cpu().numpy() - out_o).max())
            assert err <= OUT_TOL[ls.gpu.dtype], "token %d of decode_n off by %g" % (i, err)
            out_1 = twin.decode(qn[i:i + 1].cuda().contiguous(), kn[i:i + 1].cuda().contiguous(), vn[i:i + 1].cuda().contiguous())
            assert torch.equal(out_1.view(torch.int32 if dtype == "fp32" else torch.int16),
                               out_n[i:i + 1].view(torch.int32 if dtype == "fp32" else torch.int16))
        ls.check_state()
        for a, b in zip(ls.gpu.export(), twin.export()):
            assert torch.equal(a, b) or torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a, b.view(torch.int32) if b.dtype == torch.float32 else b)
    qn, kn, vn = [x.cuda() for x in random_chunk(2, nd + 1, heads, kv, d, dtype)]
    ls.step(*random_chunk(530, L, heads, kv, d, dtype))
    before = len(ls.gpu)
    with pytest.raises(B.InfMLLMError) as e:                     # one token too many: nothing is enqueued
        ls.gpu.decode_n(qn, kn, vn)
    assert e.value.code == B.ECAPACITY and len(ls.gpu) == before


def test_decode_without_max_decode_is_refused():
    s = B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, max_chunk=64)
    q, k, v = [x.cuda() for x in random_chunk(1, 64, 2, 2, 64, "bf16")]
    s.step(q, k, v)
    with pytest.raises(B.InfMLLMError) as e:
        s.decode(q[:1].contiguous(), k[:1].contiguous(), v[:1].contiguous())
    assert e.value.code == B.ECAPACITY and len(s) == 64
