"""Parity of moe_forward (HIP) against the CPU oracle, through the C ABI, in stages:
  (i)   gate logits within tolerance of the fp64 oracle;
  (ii)  the oracle's top-k and grouping applied to the GPU's own fp32 logits must reproduce
        topk_idx, counts, offsets, perm and inv bit for bit (float summation order cannot
        flip a routing decision that is taken on identical fp32 values);
  (iii) the oracle's expert + combine stage on that routing gives `out` within 2e-2;
  (iv)  end to end from raw inputs, excluding tokens whose k-th and (k+1)-th logits are closer
        than the logit tolerance.
"""
import numpy as np
import pytest

from workloads import moe

pytestmark = pytest.mark.gpu

LOGIT_TOL = 1e-4     # max |got - ref| / max |ref|: bf16 products are exact in fp32, K <= 1024 additions
OUT_TOL = 2e-2


@pytest.fixture(scope="module")
def dyn():
    import torch
    assert torch.cuda.is_available()
    import paper_1707_02402_amd as d
    return d


@pytest.fixture(scope="module")
def util():
    from tests import gpu_util
    return gpu_util


def stack(m):
    W1 = np.stack([m.expert_weights(e)[0] for e in range(m.E)])
    W2 = np.stack([m.expert_weights(e)[1] for e in range(m.E)])
    return W1, W2


def oracle_experts(oracle, m, r, W1, W2):
    """Expert + combine stage of the oracle on a given routing (token by token above its 64-use buffer)."""
    if m.k <= 64:
        return oracle.moe_experts(m.x, r.topk_idx, r.topk_w, W1, W2)
    return np.stack([oracle.moe_token(m.x[t], r.topk_w[t], [W1[e] for e in r.topk_idx[t]], [W2[e] for e in r.topk_idx[t]])
                     for t in range(m.T)])


def check_routing(oracle, m, aux):
    r = oracle.moe_route(aux["logits"], m.k)
    for name in ("topk_idx", "counts", "offsets", "perm", "inv"):
        got = aux[name]
        assert got.dtype == np.int32 and (got == getattr(r, name)).all(), name
    assert np.abs(aux["topk_w"] - r.topk_w).max() < 1e-5
    return r


@pytest.mark.parametrize("T,d,h,E,k,empty", [(300, 64, 96, 20, 3, 0.2), (257, 32, 32, 5, 5, 0.0), (1000, 128, 160, 70, 1, 0.1),
                                              (64, 96, 64, 300, 8, 0.5), (1, 32, 32, 2, 2, 0.0),
                                              (24, 32, 32, 2100, 3, 0.0),
                                              (40, 32, 32, 1500, 6, 0.0),      # 32 register-held logits per lane, 16-byte loads
                                              (33, 32, 32, 1027, 4, 0.0),      # the same with rows that are not 16-byte aligned
                                              (200, 64, 96, 64, 16, 0.0),      # k beyond the register-held uses
                                              (50, 32, 32, 12, 12, 0.0),       # k = E > 8: full softmax
                                              (90, 40, 72, 12, 3, 0.0),        # d, h multiples of 8 only
                                              (70, 64, 64, 200, 70, 0.0)])     # k > 64: several selections per lane
def test_small_layers_every_element(dyn, util, oracle, T, d, h, E, k, empty):
    m = moe.small(seed=T + E, T=T, d=d, h=h, E=E, k=k, empty_frac=empty)
    W1, W2 = stack(m)
    out, aux = util.moe_run(dyn, m, W1, W2)
    ref_logits = oracle.moe_logits(m.x, m.Wg, m.Wn, m.noise)
    assert util.normwise(aux["logits"], ref_logits) < LOGIT_TOL                      # (i)
    r = check_routing(oracle, m, aux)                                                # (ii)
    assert (r.counts[m.empty] == 0).all()
    ref = oracle_experts(oracle, m, r, W1, W2)                                        # (iii)
    assert util.normwise(out, ref) < OUT_TOL
    if k > 64:
        return
    # (iv) end to end: tokens with a clear margin between the k-th and (k+1)-th logit must route identically
    e2e = oracle.moe_forward(m.x, m.Wg, m.Wn, m.noise, W1, W2, k)
    if k < E:
        srt = np.sort(ref_logits, axis=1)[:, ::-1]
        clear = (srt[:, k - 1] - srt[:, k]) > 4 * LOGIT_TOL * np.abs(ref_logits).max()
    else:
        clear = np.ones(T, bool)
    assert clear.mean() > 0.5
    assert (np.sort(e2e.topk_idx[clear], 1) == np.sort(r.topk_idx[clear], 1)).all()
    assert util.normwise(out[clear], e2e.out[clear]) < OUT_TOL


@pytest.mark.parametrize("T,d,h,E,k", [(300, 64, 96, 20, 3), (1000, 128, 160, 70, 1), (200, 64, 96, 64, 16), (577, 64, 96, 3, 2)])
def test_permute_inside_the_operand_load_equals_the_separate_kernel(dyn, util, T, d, h, E, k):
    """Default: the first expert layer gathers token rows through the grouping; MOE_SEPARATE_PERMUTE writes the
    permuted copy with k_permute first.  Same arithmetic on the same rows: identical bits."""
    m = moe.small(seed=T + E, T=T, d=d, h=h, E=E, k=k, empty_frac=0.1 if E > 10 else 0.0)
    W1, W2 = stack(m)
    dev = util.moe_inputs_dev(m, W1, W2)
    args = (dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k)
    a = dyn.moe_forward(*args)
    b = dyn.moe_forward(*args, flags=dyn.MOE_SEPARATE_PERMUTE)
    assert (util.to_host(a) == util.to_host(b)).all()
    with pytest.raises(dyn.DynbError) as e:
        dyn.moe_forward(*args, flags=2)
    assert e.value.name == "DYNB_E_UNSUPPORTED"


def test_noiseless_gate_and_ties(dyn, util, oracle):
    """noise = NULL drops the softplus term; duplicated gate columns give exactly equal logits: lower id wins."""
    m = moe.small(seed=9, T=128, d=64, h=64, E=16, k=4)
    m.Wg[:, 8:] = m.Wg[:, :8]                    # expert e and e+8 tie on every token
    W1, W2 = stack(m)
    out, aux = util.moe_run(dyn, m, W1, W2, noise=False)
    ref_logits = oracle.moe_logits(m.x, m.Wg, None, None)
    assert util.normwise(aux["logits"], ref_logits) < LOGIT_TOL
    assert (aux["logits"][:, 8:] == aux["logits"][:, :8]).all()
    r = check_routing(oracle, m, aux)
    assert (r.topk_idx[:, 0] < 8).all() and (r.topk_idx[:, 1] == r.topk_idx[:, 0] + 8).all()
    assert util.normwise(out, oracle.moe_experts(m.x, r.topk_idx, r.topk_w, W1, W2)) < OUT_TOL


@pytest.mark.parametrize("T,d,h,E,k", [(256, 256, 32, 128, 2),      # one tile, the shortest K loop the wide kernel takes
                                        (512, 320, 32, 256, 4),      # 2 x 2 tiles, an odd number of K-chunks
                                        (768, 1024, 32, 384, 8),     # 3 x 3 tiles: dies without a token tile
                                        (2304, 256, 32, 128, 1),     # 9 token tiles: two for the first die
                                        (700, 256, 32, 128, 2)])     # two whole token tiles, 188 tokens for the 64 x 64 tiles
@pytest.mark.parametrize("noisy", [True, False])
def test_wide_gate_tiles(dyn, util, oracle, T, d, h, E, k, noisy):
    """Whole 256-token x 128-expert tiles go to the wide gate kernel (tokens behind the last whole tile, and every
    other shape in this file, to the 64 x 64 one): every logit against the oracle, with and without the noise term, routing on the GPU's logits;
    duplicated gate columns tie exactly and the lower id wins."""
    m = moe.small(seed=T + E + d, T=T, d=d, h=h, E=E, k=k)
    if not noisy:
        m.Wg[:, 64:128] = m.Wg[:, :64]           # expert e and e+64: same tile, the other expert half of a workgroup
        m.x[3, :] = 0                            # a token whose logits all tie: experts 0 .. k-1, in that order
    W1, W2 = stack(m)
    out, aux = util.moe_run(dyn, m, W1, W2, noise=noisy)
    ref_logits = oracle.moe_logits(m.x, m.Wg, m.Wn if noisy else None, m.noise if noisy else None)
    assert util.normwise(aux["logits"], ref_logits) < LOGIT_TOL
    assert np.abs(aux["logits"] - ref_logits).max() < 4 * LOGIT_TOL * np.abs(ref_logits).max()
    if not noisy:
        assert (aux["logits"][:, 64:128] == aux["logits"][:, :64]).all()
        assert (aux["logits"][3] == 0).all() and (aux["topk_idx"][3] == np.arange(k)).all()
    r = check_routing(oracle, m, aux)
    assert util.normwise(out, oracle_experts(oracle, m, r, W1, W2)) < OUT_TOL


@pytest.mark.parametrize("T,d,h,E,k,zipf", [(1536, 256, 512, 6, 2, 1.5),      # most groups beyond 256 rows, ragged rests
                                             (2048, 128, 256, 3, 1, 0.0),      # near-equal groups, short K loops
                                             (700, 256, 256, 2, 2, 0.0)])      # every token to both experts: 700 rows each
def test_crowded_experts(dyn, util, oracle, T, d, h, E, k, zipf):
    """Few experts with hundreds of rows each (groups of several full 64-row tiles that share weight tiles, and a
    ragged last tile): every output row against the oracle."""
    m = moe.small(seed=T + E + d, T=T, d=d, h=h, E=E, k=k, zipf_s=zipf)
    W1, W2 = stack(m)
    out, aux = util.moe_run(dyn, m, W1, W2)
    r = check_routing(oracle, m, aux)
    assert (r.counts >= 256).any() and (r.counts % 64 != 0).any()
    assert util.normwise(out, oracle_experts(oracle, m, r, W1, W2)) < OUT_TOL


def full_layer(dyn, util, m):
    """Runs a benchmark-size layer with per-expert generated weights; returns (out, aux, device inputs)."""
    import torch
    W1b = np.empty((m.E, m.h, m.d), np.uint16)
    W2b = np.empty((m.E, m.d, m.h), np.uint16)
    m.all_expert_weights_bits(W1b, W2b, threads=16)
    dev = util.moe_inputs_dev(m, np.zeros((1, 1, 1), np.float32), np.zeros((1, 1, 1), np.float32))
    dev["W1"] = torch.from_numpy(W1b.view(np.int16)).cuda().view(torch.bfloat16)
    dev["W2"] = torch.from_numpy(W2b.view(np.int16)).cuda().view(torch.bfloat16)
    out, aux = util.moe_run(dyn, m, dev=dev)
    out2, aux2 = util.moe_run(dyn, m, dev=dev)
    assert (out2 == out).all() and (aux2["perm"] == aux["perm"]).all()               # deterministic
    sep = dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k,
                          flags=dyn.MOE_SEPARATE_PERMUTE)
    assert (util.to_host(sep) == out).all()              # permute as its own kernel or inside the operand load: same bits
    return out, aux, dev, (W1b, W2b)


def per_token_errors(got, ref):
    """max |got - ref| / max |ref| of every token's output row."""
    den = np.abs(ref).max(axis=1)
    return np.abs(got - ref).max(axis=1) / np.where(den > 0, den, 1.0)


def test_config3_every_token(dyn, util, oracle):
    from workloads.rng import bf16_to_f32
    m = moe.config3()
    out, aux, dev, (W1b, W2b) = full_layer(dyn, util, m)
    ref_logits = oracle.moe_logits(m.x, m.Wg, m.Wn, m.noise)                         # (i) every logit
    assert util.normwise(aux["logits"], ref_logits) < LOGIT_TOL
    r = check_routing(oracle, m, aux)                                                # (ii) whole layer
    assert (r.counts[m.empty] == 0).all() and r.counts.sum() == m.A
    ref = oracle.moe_experts(m.x, r.topk_idx, r.topk_w, bf16_to_f32(W1b), bf16_to_f32(W2b))   # (iii) every token
    errs = per_token_errors(out, ref)
    assert errs.max() < OUT_TOL, (int(errs.argmax()), float(errs.max()))
    print(f"config 3: per-token error max {errs.max():.2e} median {np.median(errs):.2e}")
    load = np.sort(r.counts)[::-1].astype(np.float64)
    ok = load >= 8
    slope = np.polyfit(np.log(np.arange(1, m.E + 1)[ok]), np.log(load[ok]), 1)[0]
    assert abs(slope + 1.1) < 0.15


def config4_token_sample(r, k, min_tokens=512):
    """Tokens of config 4 whose output rows together touch every tile shape of the grouped expert layers:
    every use of 48 experts with fewer than 16 rows (one live 16-row sub-tile), of four experts with 17..63
    rows (two or four sub-tiles, ragged), and of the largest expert the first, a middle and the last 64-row
    tile (every fourth row plus the tile's first and last row); filled up with seeded random tokens."""
    counts, offsets, perm = r.counts, r.offsets, r.perm
    g = np.random.default_rng(4)
    pos = []
    tail = np.flatnonzero((counts > 0) & (counts < 16))
    tail = g.choice(tail, 48, replace=False)
    mid = np.flatnonzero((counts >= 17) & (counts <= 63))
    mid = np.concatenate([g.choice(mid[counts[mid] <= 32], 2, replace=False), g.choice(mid[counts[mid] > 32], 2, replace=False)])
    for e in np.concatenate([tail, mid]):
        pos += list(range(offsets[e], offsets[e + 1]))
    head = int(counts.argmax())
    n_tiles = (counts[head] + 63) // 64
    for tile in (0, n_tiles // 2, n_tiles - 1):
        lo = offsets[head] + 64 * tile
        hi = min(lo + 64, offsets[head + 1])
        pos += sorted(set(range(lo, hi, 4)) | {lo, hi - 1})
    tokens = set(int(perm[p]) // k for p in pos)
    T = len(r.topk_idx)
    while len(tokens) < min_tokens:
        tokens.add(int(g.integers(T)))
    return np.array(sorted(tokens)), dict(tail=tail, mid=mid, head=head, n_tiles=int(n_tiles))


def test_config4_targeted_tokens_with_empty_experts(dyn, util, oracle):
    from concurrent.futures import ThreadPoolExecutor
    m = moe.config4()
    out, aux, dev, (W1b, W2b) = full_layer(dyn, util, m)
    del W1b, W2b
    r = check_routing(oracle, m, aux)                                                # (ii) whole layer, bit-exact
    assert (r.counts[m.empty] == 0).all() and r.counts.sum() == m.A
    assert (np.sort(aux["perm"]) == np.arange(m.A)).all()
    assert (r.counts == 0).sum() >= 51 and len(m.empty) == 51
    tokens, info = config4_token_sample(r, m.k)
    assert len(tokens) >= 512 and len(info["tail"]) == 48 and info["n_tiles"] > 100
    ref_logits = oracle.moe_logits(m.x[tokens], m.Wg, m.Wn, m.noise[tokens])         # (i) the sampled rows
    assert util.normwise(aux["logits"][tokens], ref_logits) < LOGIT_TOL
    experts = np.unique(r.topk_idx[tokens])
    with ThreadPoolExecutor(16) as ex:                                               # weights regenerated per expert
        packs = dict(zip(experts.tolist(), ex.map(lambda e: m.expert_weights(int(e)), experts)))

    def one(t):
        es = [int(e) for e in r.topk_idx[t]]
        return oracle.moe_token(m.x[t], r.topk_w[t], [packs[e][0] for e in es], [packs[e][1] for e in es])

    with ThreadPoolExecutor(16) as ex:                                               # (iii) token by token
        ref = np.stack(list(ex.map(one, tokens)))
    errs = per_token_errors(out[tokens], ref)
    assert errs.max() < OUT_TOL, (int(tokens[errs.argmax()]), float(errs.max()))
    print(f"config 4: {len(tokens)} tokens through {len(experts)} experts, per-token error max {errs.max():.2e}")


def test_naive_per_use_loop_equals_batched_layer(dyn, util):
    """Results / MoE: the naive version loops over the k*b uses; same kernels, so the same bits as long as
    no group fills a 64-row tile (full tiles are multiplied with the 32x32x16 MFMA shape, which sums in
    another order)."""
    m = moe.small(seed=12, T=40, d=64, h=96, E=9, k=3, empty_frac=0.2)
    W1, W2 = stack(m)
    dev = util.moe_inputs_dev(m, W1, W2)
    a = dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k)
    b = dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, naive_stride=1)
    assert (util.to_host(a) == util.to_host(b)).all()
    m2 = moe.small(seed=13, T=400, d=96, h=288, E=6, k=2)              # groups with full tiles: tolerance
    W1, W2 = stack(m2)
    dev2 = util.moe_inputs_dev(m2, W1, W2)
    a2 = dyn.moe_forward(dev2["x"], dev2["Wg"], dev2["Wn"], dev2["noise"], dev2["W1"], dev2["W2"], m2.k)
    b2 = dyn.moe_forward(dev2["x"], dev2["Wg"], dev2["Wn"], dev2["noise"], dev2["W1"], dev2["W2"], m2.k, naive_stride=1)
    assert util.normwise(util.to_host(a2), util.to_host(b2)) < 1e-2
    with pytest.raises(dyn.DynbError):
        dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, naive_stride=-1)


def test_moe_error_paths(dyn, util):
    import torch
    m = moe.small(seed=1, T=16, d=32, h=32, E=4, k=2)
    W1, W2 = stack(m)
    dev = util.moe_inputs_dev(m, W1, W2)
    with pytest.raises(dyn.DynbError) as e:
        dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], 5)
    assert e.value.name == "DYNB_E_INVAL"
    with pytest.raises(dyn.DynbError) as e:
        dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], 2,
                        workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.name == "DYNB_E_WORKSPACE"
    with pytest.raises(dyn.DynbError) as e:
        dyn.moe_forward(dev["x"], dev["Wg"], None, dev["noise"], dev["W1"], dev["W2"], 2)
    assert e.value.name == "DYNB_E_INVAL"


def test_zero_tokens_is_a_successful_no_op(dyn):
    import torch
    d, h, E, k = 32, 32, 4, 2
    z = lambda *shape, dt=torch.bfloat16: torch.zeros(shape, dtype=dt, device="cuda")
    out = dyn.moe_forward(z(0, d), z(E, d), z(E, d), z(0, E, dt=torch.float32), z(E, h, d), z(E, d, h), k)
    assert out.shape == (0, d)


def test_every_token_to_one_expert_with_a_one_row_tail_tile(dyn, util, oracle):
    """k = 1 and one dominant gate column: a single group of 64*9 + 1 rows, every other group empty."""
    m = moe.small(seed=40, T=577, d=64, h=96, E=6, k=1)
    Wg = np.zeros_like(m.Wg)
    Wg[:, 4] = 0.0
    noise = np.full_like(m.noise, -8.0)
    noise[:, 4] = 8.0                                   # softplus(0) = ln 2: logit +-5.5, expert 4 always wins
    from dataclasses import replace
    m = replace(m, Wg=Wg, Wn=np.zeros_like(m.Wn), noise=noise)
    W1, W2 = stack(m)
    out, aux = util.moe_run(dyn, m, W1, W2)
    assert (aux["topk_idx"] == 4).all() and aux["counts"].tolist() == [0, 0, 0, 0, 577, 0]
    assert (aux["perm"] == np.arange(577)).all() and np.allclose(aux["topk_w"], 1.0)
    ref = oracle.moe_experts(m.x, aux["topk_idx"], aux["topk_w"], W1, W2)
    assert util.normwise(out, ref) < OUT_TOL


def test_layers_in_flight_on_three_streams(dyn, util):
    """Independent calls on their own streams, workspaces and outputs do not disturb each other.  The device is
    drained after the buffers are allocated: a side stream must not meet memory the default stream still uses."""
    import torch
    m = moe.config3()
    W1, W2 = stack(m)
    dev = util.moe_inputs_dev(m, W1, W2)
    args = (dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k)
    ref = dyn.moe_forward(*args)
    nb = dyn.moe_workspace_bytes(m.T, m.d, m.h, m.E, m.k)
    lanes = [dict(s=torch.cuda.Stream(), ws=torch.empty(nb, dtype=torch.uint8, device="cuda"), out=torch.empty_like(ref))
             for _ in range(3)]
    torch.cuda.synchronize()
    for i in range(9):
        ln = lanes[i % 3]
        dyn.moe_forward(*args, out=ln["out"], workspace=ln["ws"], stream=ln["s"])
    torch.cuda.synchronize()
    for ln in lanes:
        assert torch.equal(ln["out"], ref)


def test_random_small_shapes(dyn, util, oracle):
    """Seeded sweep over ragged shapes (d, h multiples of 32 only; E and T arbitrary; k up to min(E, 8))."""
    g = np.random.default_rng(2024)
    for case in range(10):
        T = int(g.integers(1, 400))
        d = int(g.choice([32, 64, 96, 160, 288]))
        h = int(g.choice([32, 96, 224, 320]))
        E = int(g.integers(2, 140))
        k = int(g.integers(1, min(E, 8) + 1))
        m = moe.small(seed=1000 + case, T=T, d=d, h=h, E=E, k=k, empty_frac=float(g.choice([0.0, 0.3])))
        W1, W2 = stack(m)
        out, aux = util.moe_run(dyn, m, W1, W2)
        shape = (case, T, d, h, E, k)
        assert util.normwise(aux["logits"], oracle.moe_logits(m.x, m.Wg, m.Wn, m.noise)) < LOGIT_TOL, shape
        r = check_routing(oracle, m, aux)
        ref = oracle.moe_experts(m.x, r.topk_idx, r.topk_w, W1, W2)
        assert util.normwise(out, ref) < OUT_TOL, shape
