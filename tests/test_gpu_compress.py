"""GPU parity: dropit_compress (through the C ABI) vs the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_13808_amd as dropit
from dropit_inputs import WORKLOADS, activation, f32_to_bf16_bits
from gpu_util import to_device, to_host
from test_oracle_select import check_selection_invariants

pytestmark = pytest.mark.gpu


def run_and_compare(x: np.ndarray, gamma: float, tag=""):
    print("compress case", tag, x.dtype, x.shape, "gamma", gamma, flush=True)
    k = oracle.keep_count(x.size, gamma)
    assert dropit.keep_count(x.size, gamma) == k
    xd = to_device(x)
    vals, idx = dropit.compress(xd, gamma)
    torch.cuda.synchronize()
    v, i = to_host(vals), to_host(idx)
    want_v, want_i = oracle.compress(x, k)
    assert i.shape == (k,) and v.shape == (k,)
    assert np.array_equal(i, want_i), tag
    assert v.tobytes() == want_v.tobytes(), tag
    return v, i


def test_config1_tiny_fc():
    w = WORKLOADS["tiny_fc"]
    x = activation(w.x_shape, w.x_dist, w.x_seed, w.dtype)
    v, i = run_and_compare(x, w.gamma, "tiny_fc")
    assert i.size == 1638


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("numel", [1, 7, 8, 9, 4095, 4097, 300003, (1 << 20) + 5, 5000011])
def test_sizes_and_ragged_tails(dtype, numel):
    x = activation((numel,), "normal", 31 + numel % 1000, dtype)
    for gamma in (0.9, 0.5):
        run_and_compare(x, gamma, "ragged")


@pytest.mark.parametrize("dist,dtype", [("normal", "bf16"), ("gelu", "bf16"), ("relu", "bf16"),
                                        ("relu", "f32"), ("gelu", "f32")])
@pytest.mark.parametrize("gamma", [0.0, 0.3, 0.8, 0.9, 0.999, 1.0])
def test_distributions_and_gammas(dist, dtype, gamma):
    x = activation((1237, 769), dist, 77, dtype)          # spans many tiles, odd row length
    run_and_compare(x, gamma, dist)


def _adversarial(n, rng):
    special = rng.standard_normal(n).astype(np.float32)
    special[::7] = np.inf
    special[1::11] = -np.inf
    special[2::13] = np.nan
    special[3::17] = -np.float32(np.nan)
    return {
        "constant": np.full(n, -1.5, np.float32),
        "zeros_mixed_sign": np.where(rng.random(n) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32),
        "two_level": np.where(rng.random(n) < 0.05, np.float32(-8.0), np.float32(0.25)).astype(np.float32),
        "few_values": rng.integers(-3, 4, n).astype(np.float32),
        "denormal": rng.integers(0, 64, n).astype(np.uint32).view(np.float32),
        "inf_nan": special,
        "ascending": np.arange(n, dtype=np.float32),
        "descending": np.arange(n, 0, -1).astype(np.float32),
    }


@pytest.mark.parametrize("n", [1000, 70001])
def test_adversarial_ties(n):
    rng = np.random.default_rng(n)
    for name, x in _adversarial(n, rng).items():
        for xx in (x, f32_to_bf16_bits(x)):
            for gamma in (0.0, 0.25, 0.5, 0.9, 0.97):
                run_and_compare(xx, gamma, name)


@pytest.mark.parametrize("name", ["vitb_fc1", "vitb_fc2", "vitdet_fc1", "vitdet_fc2", "resnet_conv3x3"])
def test_full_size_configs(name):
    w = WORKLOADS[name]
    x = activation(w.x_shape, w.x_dist, w.x_seed, w.dtype)
    v, i = run_and_compare(x, w.gamma, name)
    check_selection_invariants(x, i.size, v, i)


def _keys(t: torch.Tensor) -> torch.Tensor:
    """Magnitude keys (bit pattern with the sign cleared) of a device tensor, as int32."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).to(torch.int32) & 0x7FFF
    return t.view(torch.int32) & 0x7FFFFFFF


@pytest.mark.parametrize("dtype,mode", [("bf16", 0), ("f32", 0), ("bf16", 1)])
def test_maximum_size_properties(dtype, mode):
    """numel = 2^31 - 1, the largest tensor the int32 index allows (Sec. 3.2: the cache holds values and indices).
    The oracle's full sort is out of reach at this size, so the result is checked through the properties that
    define it, each evaluated with plain torch reductions over the input in pieces: exactly k pairs, strictly
    ascending in-range indices, vals == x[idx], every key above the threshold kept, and the ties kept being the
    first m in index order."""
    numel, gamma, piece = (1 << 31) - 1, 0.99, 1 << 28
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda:0").manual_seed(77)
    x = torch.empty(numel, dtype=tdt, device="cuda:0")
    for s in range(0, numel, piece):
        n = min(piece, numel - s)
        x[s:s + n] = torch.randn(n, device="cuda:0", dtype=torch.float32, generator=gen).to(tdt)
    x[numel - 1] = 1000.0                       # the very last element is among the largest and must be kept
    k = dropit.keep_count(numel, gamma)
    dropit.set_select_mode(mode)
    try:
        vals, idx = dropit.compress(x, gamma)
        torch.cuda.synchronize()
    finally:
        dropit.set_select_mode(0)
    assert vals.numel() == k and idx.numel() == k
    assert int(idx[0]) >= 0 and int(idx[-1]) == numel - 1
    assert bool((idx[1:] > idx[:-1]).all())
    ibits = torch.int16 if dtype == "bf16" else torch.int32
    assert bool((x[idx.long()].view(ibits) == vals.view(ibits)).all())
    kept = _keys(vals)
    t = int(kept.min())
    n_gt = n_eq = 0
    for s in range(0, numel, piece):
        kk = _keys(x[s:s + min(piece, numel - s)])
        n_gt += int((kk > t).sum())
        n_eq += int((kk == t).sum())
    m = k - n_gt
    assert 1 <= m <= n_eq
    assert int((kept > t).sum()) == n_gt and int((kept == t).sum()) == m
    seen, want_last = 0, -1
    for s in range(0, numel, piece):
        pos = torch.nonzero(_keys(x[s:s + min(piece, numel - s)]) == t).flatten()
        if seen + pos.numel() >= m:
            want_last = int(pos[m - seen - 1]) + s
            break
        seen += pos.numel()
    assert int(idx[kept == t][-1]) == want_last


def _select_path(ws: torch.Tensor) -> int:
    """White box: word 11 of the workspace's state block says how the persistent kernel found the threshold's
    key range (0 exact digit histograms, 1 sampled bracket confirmed, 2 sampled bracket missed, exact retry)."""
    return int(ws[:48].cpu().numpy().view(np.uint32)[11])


def _run_with_path(x, gamma):
    xd = to_device(x)
    ws = torch.zeros(dropit.compress_workspace_bytes(x.size, xd.dtype), dtype=torch.uint8, device="cuda:0")
    k = oracle.keep_count(x.size, gamma)
    want_v, want_i = oracle.compress(x, k)
    vals, idx = dropit.compress(xd, gamma, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(idx), want_i) and to_host(vals).tobytes() == want_v.tobytes()
    return _select_path(ws)


def test_sampled_bracket_paths():
    """Large 16-bit tensors predict the threshold's bin from a sample every workgroup reads for itself (512 pieces
    of 32 elements, one per equal stretch of the tensor at a hashed position inside it) and confirm it with exact
    counts.  All three outcomes must give the oracle's bytes: confirmed, unusable (quantile too close to an
    end), and missed -- forced here by giving exactly the sampled pieces a different scale from the rest, which
    no confidence margin can cover."""
    numel = 1 << 22
    rng = np.random.default_rng(99)
    base = rng.standard_normal(numel, dtype=np.float32)
    assert _run_with_path(f32_to_bf16_bits(base), 0.9) == 1
    assert _run_with_path(f32_to_bf16_bits(base), 0.99999) == 0          # k = 41: no usable margin
    assert _run_with_path(base, 0.9) == 0                                 # fp32 always builds the exact histograms
    nvf = numel // 8
    seg = (nvf // 4) // 512                                               # 512 pieces of 4 vectors
    sampled = np.zeros(nvf, dtype=bool)
    for i in range(512):
        h = ((i + 1) * 0x9E3779B1) & 0xFFFFFFFF
        first = (i * seg + (h >> 8) % seg) * 4
        sampled[first:first + 4] = True
    assert sampled.sum() == 2048
    scale = np.where(np.repeat(sampled, 8), np.float32(0.01), np.float32(1.0))
    assert _run_with_path(f32_to_bf16_bits(base * scale), 0.9) == 2
    scale = np.where(np.repeat(sampled, 8), np.float32(100.0), np.float32(1.0))
    assert _run_with_path(f32_to_bf16_bits(base * scale), 0.9) == 2
    # a tensor of one value: every bin of the bracket but one is empty, the ties decide everything
    assert _run_with_path(f32_to_bf16_bits(np.full(numel, 0.5, dtype=np.float32)), 0.9) in (0, 1)
    # threshold exactly between two distant bins: 40 % large, 60 % small, k at the boundary +- 1
    two = np.where(rng.random(numel) < 0.4, np.float32(8.0), np.float32(0.001)).astype(np.float32)
    n_big = int((two == 8.0).sum())
    for k in (n_big - 1, n_big, n_big + 1):
        gamma = 1.0 - (k + 0.5) / numel
        assert oracle.keep_count(numel, gamma) == k
        _run_with_path(f32_to_bf16_bits(two), gamma)


def _structured(kind, numel, rng):
    """Inputs whose values depend on the position in ways a block sample could trip over."""
    base = rng.standard_normal(numel, dtype=np.float32)
    if kind == "columns":            # every column of a 768-wide matrix has its own scale over four decades
        scale = (10.0 ** rng.uniform(-2, 2, 768)).astype(np.float32)
        return base * np.resize(scale, numel)
    if kind == "sorted":             # magnitudes grow with the index
        return np.sort(np.abs(base)) * np.where(rng.random(numel) < 0.5, np.float32(-1), np.float32(1))
    if kind == "half_zero":          # nothing but zeros in the first half
        base[: numel // 2] = 0.0
        return base
    if kind == "periodic":           # one 1 KB block in eight is a thousand times larger
        blocks = np.arange(numel) // 512
        return base * np.where(blocks % 8 == 3, np.float32(1000.0), np.float32(1.0))
    if kind == "few_values":         # five distinct magnitudes: every threshold is a massive tie
        return rng.choice(np.array([0.0, 0.25, -0.25, 1.0, -3.0, 7.0], dtype=np.float32), size=numel)
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["columns", "sorted", "half_zero", "periodic", "few_values"])
def test_large_structured_inputs(kind):
    """Large 16-bit tensors (the sampled first digit applies) with position-dependent structure, ragged tails and
    several gammas: whichever path the kernel takes, the bytes are the oracle's."""
    rng = np.random.default_rng(sum(kind.encode()))
    numel = (1 << 21) + int(rng.integers(0, 1 << 20))
    x = f32_to_bf16_bits(_structured(kind, numel, rng))
    for gamma in (0.9, 0.5, 0.97):
        path = _run_with_path(x, gamma)
        print("structured", kind, numel, gamma, "path", path, flush=True)


@pytest.mark.parametrize("numel", [(1 << 21) - 1, 1 << 21, (1 << 21) + 1, 3000017, 5 * (1 << 20) + 77])
def test_sizes_around_the_sampling_threshold(numel):
    rng = np.random.default_rng(numel)
    x = f32_to_bf16_bits(rng.standard_normal(numel, dtype=np.float32))
    expect_sampling = numel >= (1 << 21)
    for gamma in (0.8, 0.95):
        path = _run_with_path(x, gamma)
        assert path in ((0, 1, 2) if expect_sampling else (0,)), (numel, gamma, path)


def test_two_streams_at_once():
    """Two persistent selects submitted on two streams at the same time (each with its own workspace): both finish,
    both match the oracle.  The device runs them one after the other, or -- should their workgroups ever share the
    compute units -- the bounded barriers send one of them to its serial redo; either way the bytes are the same."""
    xs = [activation((3001, 700), "gelu", 71 + i, "bf16") for i in range(2)]
    want = [oracle.compress(x, oracle.keep_count(x.size, 0.9)) for x in xs]
    xd = [to_device(x) for x in xs]
    wss = [torch.empty(dropit.compress_workspace_bytes(x.size, torch.bfloat16), dtype=torch.uint8, device="cuda:0") for x in xs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(5):
        outs = []
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                outs.append(dropit.compress(xd[i], 0.9, workspace=wss[i], stream=streams[i]))
        torch.cuda.synchronize()
        for i in range(2):
            assert np.array_equal(to_host(outs[i][1]), want[i][1]) and to_host(outs[i][0]).tobytes() == want[i][0].tobytes()


def test_deterministic_and_workspace_contents_irrelevant():
    x = activation((3001, 257), "gelu", 5, "bf16")
    xd = to_device(x)
    ws = torch.empty(dropit.compress_workspace_bytes(x.size, xd.dtype), dtype=torch.uint8, device="cuda:0")
    outs = []
    for fill in (0, 255, 0x5A):
        ws.fill_(fill)
        vals, idx = dropit.compress(xd, 0.9, workspace=ws)
        torch.cuda.synchronize()
        outs.append((to_host(vals).tobytes(), to_host(idx).tobytes()))
    assert outs[0] == outs[1] == outs[2]


def test_does_not_write_past_k():
    x = activation((100000,), "normal", 9, "bf16")
    xd = to_device(x)
    k = dropit.keep_count(x.size, 0.9)
    vals = torch.full((k + 64,), 7.0, dtype=torch.bfloat16, device="cuda:0")
    idx = torch.full((k + 64,), -5, dtype=torch.int32, device="cuda:0")
    dropit.compress(xd, 0.9, vals=vals, idx=idx)
    torch.cuda.synchronize()
    assert torch.all(idx[k:] == -5) and torch.all(vals[k:] == 7.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_separate_kernel_mode_matches_oracle(dtype):
    """Mode 1 (ordinary kernels, the graph-capturable form) gives the same bytes as the oracle."""
    dropit.set_select_mode(1)
    try:
        for numel in (9, 4097, 300003, (1 << 20) + 5):
            x = activation((numel,), "relu", 500 + numel % 97, dtype)
            for gamma in (0.9, 0.3):
                run_and_compare(x, gamma, "separate-kernels")
        w = WORKLOADS["vitb_fc1"]
        if dtype == "bf16":
            run_and_compare(activation(w.x_shape, w.x_dist, w.x_seed, w.dtype), w.gamma, "separate-kernels vitb_fc1")
    finally:
        dropit.set_select_mode(0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode,label", [(3, "forced serial redo"), (2, "cooperative launch")])
def test_other_select_modes_match_oracle(dtype, mode, label):
    """Mode 3 gives the grid barriers zero patience, so (nearly) every workgroup gives up and the last
    one to leave redoes the selection alone; mode 2 launches the same kernel cooperatively.  Both
    must give the oracle's bytes, and every kernel exits normally."""
    dropit.set_select_mode(mode)
    try:
        for numel in (3, 9, 4097, 300003, (1 << 20) + 5):
            x = activation((numel,), "relu", 600 + numel % 89, dtype)
            for gamma in (0.9, 0.3):
                run_and_compare(x, gamma, label)
        if dtype == "bf16":
            w = WORKLOADS["vitb_fc1"]
            run_and_compare(activation(w.x_shape, w.x_dist, w.x_seed, w.dtype), w.gamma, label + " vitb_fc1")
    finally:
        dropit.set_select_mode(0)


@pytest.mark.parametrize("mode", [0, 1])
def test_select_in_a_hip_graph(mode):
    """Both ordinary-launch forms replay correctly from a captured graph (no memset nodes inside)."""
    x = activation((123457,), "gelu", 77, "bf16")
    xd = to_device(x)
    k = dropit.keep_count(x.size, 0.9)
    vals = torch.zeros(k, dtype=torch.bfloat16, device="cuda:0")
    idx = torch.zeros(k, dtype=torch.int32, device="cuda:0")
    ws = torch.empty(dropit.compress_workspace_bytes(x.size, xd.dtype), dtype=torch.uint8, device="cuda:0")
    want_v, want_i = oracle.compress(x, k)
    dropit.set_select_mode(mode)
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            dropit.compress(xd, 0.9, vals=vals, idx=idx, workspace=ws)       # warm-up outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            dropit.compress(xd, 0.9, vals=vals, idx=idx, workspace=ws)
        for replay in range(3):
            vals.zero_()
            idx.zero_()
            ws.fill_(replay * 37)                                            # eager work between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(to_host(idx), want_i), replay
            assert to_host(vals).tobytes() == want_v.tobytes(), replay
    finally:
        dropit.set_select_mode(0)


@pytest.mark.parametrize("numel", [123457, (1 << 21) + 4099])
def test_graph_replays_over_changing_inputs_with_an_untouched_workspace(numel):
    """The real use of a captured training step: the same graph (hence the same kernel arguments, the persistent
    kernel's per-call number included) replayed while the activations change in place and nobody touches the
    workspace in between.  Every replay must give the oracle's bytes for the input it saw; the larger size takes
    the sampled form."""
    dists = ["gelu", "normal", "relu", "gelu"]
    xs = [activation((numel,), d, 90 + i, "bf16") for i, d in enumerate(dists)]
    xs[3] = f32_to_bf16_bits(np.random.default_rng(5).standard_normal(numel, dtype=np.float32) * 1000.0)   # the threshold moves far away
    k = dropit.keep_count(numel, 0.9)
    want = [oracle.compress(x, k) for x in xs]
    xd = to_device(xs[0])
    vals = torch.zeros(k, dtype=torch.bfloat16, device="cuda:0")
    idx = torch.zeros(k, dtype=torch.int32, device="cuda:0")
    ws = torch.empty(dropit.compress_workspace_bytes(numel, xd.dtype), dtype=torch.uint8, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dropit.compress(xd, 0.9, vals=vals, idx=idx, workspace=ws)           # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        dropit.compress(xd, 0.9, vals=vals, idx=idx, workspace=ws)
    for replay in range(8):
        which = replay % len(xs)
        xd.copy_(to_device(xs[which]))                                       # new activations, in place
        vals.zero_()
        idx.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(to_host(idx), want[which][1]), (replay, which)
        assert to_host(vals).tobytes() == want[which][0].tobytes(), (replay, which)


def test_forced_redo_is_reported():
    """White box: word 14 of the state block says whether the grid barriers gave up and the last workgroup redid
    the selection alone (mode 3 forces that); an ordinary call reports 0."""
    x = activation((300003,), "gelu", 17, "bf16")
    xd = to_device(x)
    k = oracle.keep_count(x.size, 0.9)
    want_v, want_i = oracle.compress(x, k)
    for mode, expect in ((0, 0), (3, 1), (0, 0)):
        ws = torch.full((dropit.compress_workspace_bytes(x.size, xd.dtype),), 0xA5, dtype=torch.uint8, device="cuda:0")
        dropit.set_select_mode(mode)
        try:
            vals, idx = dropit.compress(xd, 0.9, workspace=ws)
            torch.cuda.synchronize()
        finally:
            dropit.set_select_mode(0)
        assert np.array_equal(to_host(idx), want_i) and to_host(vals).tobytes() == want_v.tobytes()
        assert int(ws[:64].cpu().numpy().view(np.uint32)[14]) == expect, mode


def _state_words(ws: torch.Tensor) -> np.ndarray:
    return ws[:64].cpu().numpy().view(np.uint32)


def _run_with_state(x, gamma):
    xd = to_device(x)
    ws = torch.zeros(dropit.compress_workspace_bytes(x.size, xd.dtype), dtype=torch.uint8, device="cuda:0")
    k = oracle.keep_count(x.size, gamma)
    want_v, want_i = oracle.compress(x, k)
    vals, idx = dropit.compress(xd, gamma, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(idx), want_i) and to_host(vals).tobytes() == want_v.tobytes()
    st = _state_words(ws)
    return dict(path=int(st[11]), groups=int(st[10] & 0xFFFF), redo=int(st[14]), staged=int(st[15]))


@pytest.mark.parametrize("name", ["vitb_fc1", "vitb_fc2", "vitdet_fc2", "resnet_conv3x3"])
def test_benchmark_tensors_are_read_once(name):
    """White box: on the benchmark tensors the sampled bracket is confirmed and EVERY workgroup compacts from the
    candidates it staged in LDS during its one pass over x (word 15 of the state block counts them, the low half
    of word 10 the workgroups)."""
    w = WORKLOADS[name]
    s = _run_with_state(activation(w.x_shape, w.x_dist, w.x_seed, w.dtype), w.gamma)
    print("staged", name, s, flush=True)
    assert s["path"] == 1 and s["redo"] == 0
    assert s["groups"] > 1 and s["staged"] == s["groups"]


@pytest.mark.parametrize("numel,gamma", [((9 << 20) + 1234, 0.9), (3 * (1 << 22) + 8 * 77, 0.8), (20000011, 0.95)])
def test_staging_overflow_falls_back_per_workgroup(numel, gamma):
    """Values that bunch up along the tensor: the largest eighth of a normal sample sits (shuffled) in the first
    eighth of the tensor, so the value histogram is the ordinary one (the sampled bracket is usable) but the
    workgroups that own that stretch find most of their elements candidates, more than their LDS segments hold, and
    take the two-read form, while the others stage theirs.  Same bytes either way."""
    rng = np.random.default_rng(numel % 1000)
    base = rng.standard_normal(numel, dtype=np.float32)
    order = np.argsort(-np.abs(base), kind="stable")
    head = numel // 8
    out = np.empty_like(base)
    out[:head] = base[rng.permutation(order[:head])]
    out[head:] = base[rng.permutation(order[head:])]
    s = _run_with_state(f32_to_bf16_bits(out), gamma)
    print("overflow", numel, gamma, s, flush=True)
    assert s["path"] == 1 and s["redo"] == 0
    assert 0 < s["staged"] < s["groups"]


@pytest.mark.parametrize("numel", [(1 << 21), (1 << 21) + 8 * 1000 + 3, 2500000, 7 * (1 << 20) + 5])
@pytest.mark.parametrize("dist", ["normal", "relu", "gelu"])
def test_staged_form_sizes_and_ragged_ends(numel, dist):
    """Chunk and wavefront ranges that end inside a block, inside a lane's pair of vectors, and with a ragged
    (numel % 8) tail, for the three activation shapes and three gammas."""
    x = activation((numel,), dist, 40 + numel % 97, "bf16")
    for gamma in (0.9, 0.8, 0.6):
        s = _run_with_state(x, gamma)
        print("staged sizes", numel, dist, gamma, s, flush=True)


@pytest.mark.parametrize("dtype,numel", [("f32", 32767), ("f32", 32768), ("f32", 32771), ("f32", 32776),
                                         ("bf16", 65535), ("bf16", 65536), ("bf16", 65543), ("bf16", 65544),
                                         ("bf16", 20000), ("f32", 1025), ("bf16", 8193)])
def test_one_workgroup_form_and_its_size_limit(dtype, numel):
    """Tensors of up to 8 x 1024 16-byte vectors take the one-workgroup kernel (registers only, no workspace);
    one element more takes the persistent kernel.  Same bytes on either side of the limit."""
    for dist, gamma in (("normal", 0.9), ("relu", 0.3), ("gelu", 0.75)):
        run_and_compare(activation((numel,), dist, 11 + numel % 13, dtype), gamma, "small")


@pytest.mark.parametrize("dtype,numel,mode", [("bf16", 3000017, 0), ("bf16", 300003, 0), ("f32", 300003, 0), ("bf16", 300003, 1),
                                              ("f32", 20000, 0)])
def test_nothing_is_written_outside_the_workspace_and_the_outputs(dtype, numel, mode):
    """Canaries: the select's workspace and both outputs sit inside poisoned buffers of exactly the advertised size."""
    x = activation((numel,), "gelu", 23, dtype)
    xd = to_device(x)
    k = dropit.keep_count(numel, 0.9)
    guard, pattern = 4096, 0x3C

    def guarded(nbytes):
        size = (nbytes + 255) // 256 * 256
        whole = torch.full((guard + size + guard,), pattern, dtype=torch.uint8, device="cuda:0")
        lo = (-whole.data_ptr()) % 256 + 2048
        return whole, lo, whole[lo:lo + nbytes]

    w_ws, lo_ws, ws = guarded(dropit.compress_workspace_bytes(numel, xd.dtype))
    w_v, lo_v, vb = guarded(k * xd.element_size())
    w_i, lo_i, ib = guarded(k * 4)
    dropit.set_select_mode(mode)
    try:
        vals, idx = dropit.compress(xd, 0.9, vals=vb.view(xd.dtype), idx=ib.view(torch.int32), workspace=ws)
        torch.cuda.synchronize()
    finally:
        dropit.set_select_mode(0)
    for whole, lo, inner in ((w_ws, lo_ws, ws), (w_v, lo_v, vb), (w_i, lo_i, ib)):
        assert bool((whole[:lo] == pattern).all()) and bool((whole[lo + inner.numel():] == pattern).all())
    want_v, want_i = oracle.compress(x, k)
    assert np.array_equal(to_host(idx), want_i) and to_host(vals).tobytes() == want_v.tobytes()
