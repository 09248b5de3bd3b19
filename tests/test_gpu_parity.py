"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Tolerances: max|gpu-oracle|/max|oracle| <= 1e-4 for forward outputs and
<= 1e-3 for every gradient (fp32 arithmetic on the GPU, fp64 in the oracle)."""
import numpy as np
import pytest

from paper_1604_01946_amd.inputs import CONFIGS, Config, make_inputs
import parity
from parity import oracle_results, assert_close, FWD_TOL, BWD_TOL

pytestmark = pytest.mark.gpu

FWD = ("y", "hT", "cT")
BWD = ("dx", "dh0", "dc0", "dW", "dR", "db")


def _mods():
    import torch
    from paper_1604_01946_amd import binding, runner
    assert torch.cuda.is_available()
    return torch, binding, runner


def run_case(cfg, seed, flags, backward=True, with_states=True, with_dstates=True, poison=True):
    torch, binding, runner = _mods()
    d, ref = oracle_results(cfg, seed, with_states, with_dstates, backward)
    r = runner.LstmRunner(cfg.dims, d, with_states=with_states, with_dstates=with_dstates)
    if poison:
        r.poison()
    print(f"case {cfg.dims} seed={seed} flags={flags} bwd={backward}", flush=True)
    binding.check(r.forward(flags=flags), "lstm_forward")
    torch.cuda.synchronize()
    e = assert_close(r.fwd_outputs(), ref, FWD, FWD_TOL, f"fwd {cfg.dims} flags={flags}")
    if backward:
        bflags = flags
        if flags == binding.LSTM_PATH_PERSISTENT and binding.lstm_auto_path(*cfg.dims, 1) != flags:
            bflags = 0  # the persistent backward does not take this shape: use the automatic choice
        binding.check(r.backward(flags=bflags), "lstm_backward")
        torch.cuda.synchronize()
        e.update(assert_close(r.bwd_outputs(), ref, BWD, BWD_TOL, f"bwd {cfg.dims} flags={flags}"))
    print("  errors:", {k: f"{v:.2e}" for k, v in e.items()}, flush=True)
    print("  element-wise relative (floor 1e-6 of the scale):", {k: f"{parity.last_relerr[k]:.2e}" for k in e}, flush=True)
    return r, ref


# ------------------------------------------------------------------ GEMM alone
def _gemm_case(M, N, K, layout, scratch_bytes=None):
    """layout: first letter A (N: [M][K], T: [K][M]), second letter B (N: [K][N], T: [N][K]).
    scratch_bytes: run lstm_gemm_f32_ws with a scratch buffer of that size (0: a NULL buffer)."""
    torch, binding, _ = _mods()
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = rng.standard_normal((K, N)).astype(np.float32)
    ref = A.astype(np.float64) @ Bm.astype(np.float64)
    dev = "cuda:0"
    if layout[0] == "T":
        At = torch.from_numpy(np.ascontiguousarray(A.T)).to(dev); sAm, sAk = 1, M
    else:
        At = torch.from_numpy(A).to(dev); sAm, sAk = K, 1
    if layout[1] == "T":
        Bt = torch.from_numpy(np.ascontiguousarray(Bm.T)).to(dev); sBk, sBn = 1, K
    else:
        Bt = torch.from_numpy(Bm).to(dev); sBk, sBn = N, 1
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    if scratch_bytes is None:
        run = lambda acc: binding.lstm_gemm_f32(M, N, K, At, sAm, sAk, Bt, sBk, sBn, C, N, acc)
    else:
        scratch = torch.full((max(scratch_bytes // 4, 1),), float("nan"), dtype=torch.float32, device=dev) if scratch_bytes else None
        run = lambda acc: binding.lstm_gemm_f32_ws(M, N, K, At, sAm, sAk, Bt, sBk, sBn, C, N, acc, scratch, scratch_bytes)
    binding.check(run(0), "gemm")
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    tol = 2e-6 * max(1.0, (K / 512.0) ** 0.5)  # fp32 sums of K products: rounding grows like sqrt(K)
    assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) < tol
    binding.check(run(1), "gemm acc")
    torch.cuda.synchronize()
    assert np.max(np.abs(C.cpu().numpy() - 2 * ref)) / np.max(np.abs(ref)) < 2 * tol
    if scratch_bytes:  # repeatable bit for bit (the partial tiles are added in a fixed order)
        binding.check(run(0), "gemm")
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), got)


# K a multiple of 16 with 16-byte aligned rows takes the direct-to-LDS kernel (1, 2, 3, 4 and many
# k-tiles, ragged M and N), everything else the register-staged one
@pytest.mark.parametrize("M,N,K", [(64, 64, 16), (128, 128, 64), (200, 136, 72), (33, 17, 5), (6400, 2048, 512),
                                   (1, 1, 1), (257, 129, 130), (256, 384, 48), (100, 260, 32), (96, 68, 16)])
@pytest.mark.parametrize("layout", ["NT", "NN", "TN", "TT"])
def test_gemm_matches_numpy(M, N, K, layout):
    _gemm_case(M, N, K, layout)


# The tile (128 x 128 or 64 x 64) follows how the tiles fill the 256 CUs: half the CUs in large tiles, exactly one large
# tile per CU, a CU in eight with two, two per CU, and large tiles of which a quarter is empty (M = 192).
@pytest.mark.parametrize("M,N,K", [(256, 8192, 64), (256, 16384, 32), (384, 12288, 32), (512, 16384, 32), (192, 16384, 48)])
@pytest.mark.parametrize("layout", ["NT", "TN"])
def test_gemm_tile_choice(M, N, K, layout):
    _gemm_case(M, N, K, layout)


# Products whose tiles do not fill the chip evenly, with a scratch buffer for K slices: the shapes of the time-batched
# products at T*B = 1600 rows (a last round of few tiles; fewer tiles than places), a ragged last tile row, a product
# with whole rounds only (nothing to cut), too small a buffer (fewer slices, then none) and no buffer.
@pytest.mark.parametrize("M,N,K,scratch", [(1600, 8192, 512, 64 << 20), (1600, 2048, 2048, 64 << 20), (1610, 8192, 256, 64 << 20),
                                           (1536, 8192, 128, 64 << 20), (1600, 8192, 512, 3 << 20), (1600, 8192, 512, 1 << 20),
                                           (1600, 2048, 2048, 0), (200, 136, 64, 1 << 20)])
@pytest.mark.parametrize("layout", ["NT", "NN", "TN"])
def test_gemm_with_k_slices(M, N, K, scratch, layout):
    _gemm_case(M, N, K, layout, scratch_bytes=scratch)


@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (6400, 2048, 512), (256, 384, 48), (100, 260, 32)])
@pytest.mark.parametrize("layout", ["NT", "NN", "TN", "TT"])
def test_gemm_register_staged_kernel(M, N, K, layout, knobs):
    knobs(LSTM_GEMM_STAGED="1")
    _gemm_case(M, N, K, layout)


# ------------------------------------------------------------------ the five measured shapes
PATHS_ALL = [0, 1, 2, 3, 4, 5, 6]


# Hidden sizes below 512 that the persistent kernels do not take run zero-padded to the next one that they do, on
# every path; LSTM_NO_PAD=1 runs the shape as given, which is what exercises the ragged tiles of the per-step kernels.
# cfg1 itself is among the shapes that run a whole pass in one workgroup (automatic choice and step path):
# LSTM_MICRO=0 puts it back on the per-step kernels.
@pytest.mark.parametrize("variant", ["default", "per_step", "as_given"])
@pytest.mark.parametrize("flags", PATHS_ALL)
def test_cfg1_all_paths(flags, variant, knobs):
    _, binding, _ = _mods()
    if variant == "per_step":
        knobs(LSTM_MICRO="0")
    if variant == "as_given":
        knobs(LSTM_NO_PAD="1", LSTM_MICRO="0")
    cfg = CONFIGS["cfg1"]
    if flags == 6 and binding.lstm_auto_path(*cfg.dims, 0) != 6:
        # H = 32 as given has no persistent kernel: forcing that path must be refused, not run on something else
        r = _mods()[2].LstmRunner(cfg.dims, make_inputs(cfg, 0))
        assert r.forward(flags=6) == binding.LSTM_UNSUPPORTED
        return
    run_case(cfg, 0, flags)
    run_case(cfg, 1, flags)


@pytest.mark.parametrize("flags", [0, 4])
def test_cfg2_forward(flags):
    run_case(CONFIGS["cfg2"], 0, flags, backward=False)


@pytest.mark.parametrize("flags", [0, 4, 5, 6])
def test_cfg3_forward_backward(flags):
    run_case(CONFIGS["cfg3"], 0, flags)


def test_cfg3_second_seed():
    """Guard against anything fitted to seed 0: the measured shape once more with other inputs."""
    run_case(CONFIGS["cfg3"], 1, 0)


@pytest.mark.parametrize("flags", [0, 4], ids=["auto", "step"])
def test_cfg4_large_hidden(flags):
    """Full size: the one-layer persistent kernels (automatic path), and the step kernels that stream R every step
    (split-K backward) at the size they were built for."""
    run_case(CONFIGS["cfg4"], 0, flags)


@pytest.mark.parametrize("flags", [0, 4, 6])
def test_cfg5_small_batch_long_sequence(flags):
    run_case(CONFIGS["cfg5"], 0, flags, with_states=False, with_dstates=False)


def test_cfg5_on_the_narrow_kernels(knobs):
    """B = 1 runs on the kernels whose exchanged values are their own flags; LSTM_TINY=0 keeps the counter-based ones."""
    knobs(LSTM_TINY="0")
    run_case(CONFIGS["cfg5"], 0, 6, with_states=False, with_dstates=False)


# a single sequence: every hidden size of the flag-in-data kernels, I != H (input product and input gradient as batched
# products), one layer, one step, a stack of eight layers (512 waves), with and without initial / final states
SINGLE = [
    Config("s128", L=1, T=9, B=1, I=128, H=128, state_std=0.3, dstate_std=0.3),
    Config("s128i", L=3, T=6, B=1, I=40, H=128, state_std=0.3, dstate_std=0.3),
    Config("s256T1", L=2, T=1, B=1, I=256, H=256, state_std=0.3, dstate_std=0.3),
    Config("s256T2", L=2, T=2, B=1, I=256, H=256, state_std=0.3, dstate_std=0.3),
    Config("s256T3", L=1, T=3, B=1, I=256, H=256, state_std=0.3, dstate_std=0.3),
    Config("s512", L=2, T=7, B=1, I=512, H=512, state_std=0.3, dstate_std=0.3),
    Config("s512i", L=4, T=5, B=1, I=72, H=512, state_std=0.3, dstate_std=0.3),
    Config("s128L8", L=8, T=4, B=1, I=128, H=128, state_std=0.3, dstate_std=0.3),
    Config("s512L8", L=8, T=3, B=1, I=512, H=512, state_std=0.3, dstate_std=0.3),  # every CU holds one workgroup of 8 waves
]


@pytest.mark.parametrize("cfg", SINGLE, ids=[c.name for c in SINGLE])
@pytest.mark.parametrize("with_states", [True, False])
def test_single_sequence(cfg, with_states):
    _, binding, _ = _mods()
    run_case(cfg, 5, binding.LSTM_PATH_PERSISTENT, with_states=with_states, with_dstates=with_states)


# ------------------------------------------------------------------ persistent path: every shape class it takes
PERS = [
    Config("p128", L=2, T=5, B=16, I=40, H=128, state_std=0.3, dstate_std=0.3),
    Config("p128L8", L=8, T=4, B=7, I=128, H=128, state_std=0.3, dstate_std=0.3),
    Config("p256b1", L=2, T=12, B=1, I=256, H=256, state_std=0.3, dstate_std=0.3),
    Config("p256b20", L=3, T=6, B=20, I=64, H=256, state_std=0.3, dstate_std=0.3),
    Config("p512b33", L=2, T=5, B=33, I=72, H=512, state_std=0.3, dstate_std=0.3),
    Config("p512b64", L=4, T=7, B=64, I=512, H=512, state_std=0.3, dstate_std=0.3),
    Config("p512L1", L=1, T=9, B=48, I=512, H=512, state_std=0.3, dstate_std=0.3),
    # batches above 64 rows run as slices of 64, one launch per slice (full, ragged and nearly empty last slice)
    Config("p512b128", L=2, T=4, B=128, I=64, H=512, state_std=0.3, dstate_std=0.3),
    Config("p256b130", L=3, T=3, B=130, I=256, H=256, state_std=0.3, dstate_std=0.3),
    Config("p128b65", L=2, T=3, B=65, I=24, H=128, state_std=0.3, dstate_std=0.3),
    Config("p128b512", L=1, T=2, B=512, I=16, H=128, state_std=0.3, dstate_std=0.3),   # 8 slices side by side
    Config("p128b1100", L=1, T=2, B=1100, I=16, H=128, state_std=0.3, dstate_std=0.3),  # 18 slices: 16 side by side, then 2
    Config("p512T1", L=4, T=1, B=64, I=512, H=512, state_std=0.3, dstate_std=0.3),     # a single step
]


def test_persistent_many_slices():
    """A batch of many 64-row slices (beyond the 2048 rows that were once the limit of the persistent path), ragged last slice."""
    _, binding, _ = _mods()
    cfg = Config("p128b2100", L=2, T=3, B=2100, I=40, H=128, state_std=0.5, dstate_std=0.5)
    assert binding.lstm_auto_path(*cfg.dims, 0) == binding.LSTM_PATH_PERSISTENT
    assert binding.lstm_auto_path(*cfg.dims, 1) == binding.LSTM_PATH_PERSISTENT
    run_case(cfg, 21, 0)


@pytest.mark.parametrize("cfg", PERS, ids=[c.name for c in PERS])
@pytest.mark.parametrize("with_states", [True, False])
def test_persistent_shapes(cfg, with_states):
    _, binding, _ = _mods()
    assert binding.lstm_auto_path(*cfg.dims, 0) == binding.LSTM_PATH_PERSISTENT
    run_case(cfg, 11, binding.LSTM_PATH_PERSISTENT, with_states=with_states, with_dstates=with_states)


# Large hidden sizes: the one-layer-per-launch persistent kernels (recurrent matrix spread over all CUs)
LARGE = [
    Config("l1024b32", L=2, T=5, B=32, I=96, H=1024, state_std=0.3, dstate_std=0.3),
    Config("l1024b7", L=1, T=4, B=7, I=1024, H=1024, state_std=0.3, dstate_std=0.3),
    Config("l2048b32", L=2, T=4, B=32, I=256, H=2048, state_std=0.3, dstate_std=0.3),
    Config("l2048b5", L=1, T=3, B=5, I=64, H=2048, state_std=0.3, dstate_std=0.3),
    Config("l2048T1", L=2, T=1, B=1, I=2048, H=2048, state_std=0.3, dstate_std=0.3),   # a single step, a single row
    Config("l1024T1", L=1, T=1, B=32, I=16, H=1024, state_std=0.3, dstate_std=0.3),
    # H = 1024 above 32 rows: slices of 32 side by side (two forward, four backward) and in further launches
    Config("l1024b64", L=2, T=4, B=64, I=128, H=1024, state_std=0.3, dstate_std=0.3),
    Config("l1024b33", L=1, T=3, B=33, I=1024, H=1024, state_std=0.3, dstate_std=0.3),
    Config("l1024b100", L=2, T=3, B=100, I=64, H=1024, state_std=0.3, dstate_std=0.3),
    Config("l1024b128", L=1, T=2, B=128, I=32, H=1024, state_std=0.3, dstate_std=0.3),
    Config("l1024b160", L=1, T=2, B=160, I=48, H=1024, state_std=0.3, dstate_std=0.3),   # five slices: a second backward launch
    Config("l1024b300", L=1, T=2, B=300, I=32, H=1024, state_std=0.3, dstate_std=0.3),   # ten slices
    # H = 2048 above 32 rows: one slice fills the chip, the slices run one after the other
    Config("l2048b40", L=1, T=2, B=40, I=64, H=2048, state_std=0.3, dstate_std=0.3),
    Config("l2048b70", L=2, T=2, B=70, I=32, H=2048, state_std=0.3, dstate_std=0.3),
]


@pytest.mark.parametrize("cfg", LARGE, ids=[c.name for c in LARGE])
@pytest.mark.parametrize("with_states", [True, False])
def test_persistent_large_hidden(cfg, with_states):
    _, binding, _ = _mods()
    assert binding.lstm_auto_path(*cfg.dims, 0) == binding.LSTM_PATH_PERSISTENT
    assert binding.lstm_auto_path(*cfg.dims, 1) == binding.LSTM_PATH_PERSISTENT
    run_case(cfg, 12, binding.LSTM_PATH_PERSISTENT, with_states=with_states, with_dstates=with_states)


# H = 1024 with one or two slices cuts the backward tiles' K over the idle CUs; LSTM_LARGE_KSPLIT=0 keeps one workgroup
# per tile covered there.
@pytest.mark.parametrize("name", ["l1024b32", "l1024b7", "l1024b64", "l1024b33"])
def test_large_hidden_whole_tiles_backward(name, knobs):
    knobs(LSTM_LARGE_KSPLIT="0")
    run_case(next(c for c in LARGE if c.name == name), 14, 0)


# H = 2048 runs forward on the kernel with two alternating chains of 16 rows per slice; LSTM_LARGE_PP=0 keeps the
# one-chain kernel (the one the other cells and H = 1024 use)
@pytest.mark.parametrize("name", ["l2048b32", "l2048b5", "l2048b40", "l2048T1"])
def test_large_hidden_one_chain_forward(name, knobs):
    _, binding, _ = _mods()
    knobs(LSTM_LARGE_PP="0")
    cfg = next(c for c in LARGE if c.name == name)
    run_case(cfg, 12, binding.LSTM_PATH_PERSISTENT, with_states=True, with_dstates=True)


# Stacks deeper than the chip holds at once (L * H/8 workgroups > CUs): groups of consecutive layers, one launch each
DEEP = [
    Config("d512L8", L=8, T=5, B=64, I=512, H=512, state_std=0.3, dstate_std=0.3),      # 4 + 4, x multiplied in the kernel
    Config("d512L5", L=5, T=4, B=40, I=72, H=512, state_std=0.3, dstate_std=0.3),       # 4 + 1, x projected by a GEMM
    Config("d512L6b8", L=6, T=6, B=8, I=512, H=512, state_std=0.3, dstate_std=0.3),     # narrow kernels, 4 + 2
    Config("d256L9b130", L=9, T=3, B=130, I=256, H=256, state_std=0.3, dstate_std=0.3),  # 8 + 1, three batch slices
    Config("d128L17", L=17, T=3, B=33, I=24, H=128, state_std=0.3, dstate_std=0.3),     # 16 + 1
]


@pytest.mark.parametrize("cfg", DEEP, ids=[c.name for c in DEEP])
@pytest.mark.parametrize("with_states", [True, False])
def test_persistent_layer_groups(cfg, with_states):
    torch, binding, _ = _mods()
    assert binding.lstm_auto_path(*cfg.dims, 0) == binding.LSTM_PATH_PERSISTENT
    assert binding.lstm_auto_path(*cfg.dims, 1) == binding.LSTM_PATH_PERSISTENT
    r, ref = run_case(cfg, 13, binding.LSTM_PATH_PERSISTENT, with_states=with_states, with_dstates=with_states)
    # an inference call (no reserve) hands the hidden states from group to group through the workspace
    y_train = r.y.clone()
    r.y.fill_(float("nan"))
    binding.check(r.forward(flags=binding.LSTM_PATH_PERSISTENT, inference=True))
    torch.cuda.synchronize()
    assert torch.equal(r.y, y_train)


# ------------------------------------------------------------------ persistent path: kernel variants and the slow protocol
VARIANTS = [
    {"LSTM_FWD_NARROW": "1", "LSTM_BWD_NARROW": "1"},                      # 16x16x4 kernels at B > 32
    {"LSTM_FWD_NARROW": "1", "LSTM_BWD_NARROW": "1", "LSTM_CHAINS": "2"},  # two independent batch chains
    {"LSTM_FULL_FENCES": "1"},                                             # release/acquire fences on every step
    {"LSTM_FWD_BATCHED_INPUT": "1"},                                       # layer 0's input product as one GEMM although I == H
    {"LSTM_FWD_NARROW": "0", "LSTM_BWD_NARROW": "0"},                      # wide kernels also where slices of 16 / 32 rows on the narrow ones would fit
    {"LSTM_PINGPONG": "0"},                                                # one chain of 64 rows per slice instead of two alternating chains of 32
]


@pytest.mark.parametrize("env", VARIANTS, ids=["narrow", "chains2", "fullfences", "batched_input", "wide", "one_chain"])
@pytest.mark.parametrize("cfg", [PERS[3], PERS[4], PERS[5]], ids=["p256b20", "p512b33", "p512b64"])
def test_persistent_variants(cfg, env, knobs):
    """The alternative kernels and the fence-based protocol must give the oracle's answer too; the
    default path must give bit-identical results to the fence-based one (same arithmetic, only the
    synchronisation differs), which cross-checks the fast flag protocol."""
    torch, binding, runner = _mods()
    for k, v in env.items():
        knobs(**{k: v})
    r, ref = run_case(cfg, 11, binding.LSTM_PATH_PERSISTENT)
    if "LSTM_FULL_FENCES" in env:
        slow = {k: getattr(r, k).clone() for k in FWD + BWD}
        knobs(LSTM_FULL_FENCES=None)
        r.poison()
        binding.check(r.forward(flags=binding.LSTM_PATH_PERSISTENT))
        binding.check(r.backward(flags=binding.LSTM_PATH_PERSISTENT))
        torch.cuda.synchronize()
        for k in FWD + BWD:
            assert torch.equal(slow[k], getattr(r, k)), k


@pytest.mark.parametrize("next_path", [6, 4], ids=["persistent", "step"])
def test_watchdog_expires_and_reports(knobs, next_path):
    """A spin limit of 1 makes the waits of the persistent kernels give up at once (forced from the
    host; the kernels still run to completion).  The next call, on whatever path, must report
    LSTM_INTERNAL once, launch nothing, and the call after it must work again."""
    torch, binding, runner = _mods()
    cfg = PERS[5]
    d, ref = oracle_results(cfg, 11)
    r = runner.LstmRunner(cfg.dims, d)
    knobs(LSTM_SPIN_LIMIT="1")
    st = r.forward(flags=binding.LSTM_PATH_PERSISTENT)
    torch.cuda.synchronize()          # the kernel drained
    assert st == binding.LSTM_OK      # the expiry is seen by the host only afterwards
    r.y.fill_(float("nan"))
    st2 = r.forward(flags=next_path)
    torch.cuda.synchronize()
    if st2 == binding.LSTM_OK:
        pytest.skip("no wait expired with a spin limit of 1 (every flag was already set when polled)")
    assert st2 == binding.LSTM_INTERNAL
    assert torch.isnan(r.y).all()     # the reporting call launched nothing
    knobs(LSTM_SPIN_LIMIT=None)
    binding.check(r.forward(flags=next_path))
    torch.cuda.synchronize()
    assert_close(r.fwd_outputs(), ref, FWD, FWD_TOL)


# ------------------------------------------------------------------ ragged / odd shapes, several tiles
ODD = [
    Config("odd1", L=2, T=3, B=5, I=24, H=40, state_std=0.5, dstate_std=0.5),
    Config("odd2", L=3, T=4, B=3, I=7, H=30, state_std=0.5, dstate_std=0.5),     # H, I not multiples of 4
    Config("odd3", L=2, T=5, B=70, I=36, H=100, state_std=0.5, dstate_std=0.5),  # two batch tiles, ragged tail
    Config("odd4", L=1, T=1, B=1, I=1, H=1, state_std=0.5, dstate_std=0.5),
    Config("odd5", L=2, T=6, B=33, I=130, H=264, state_std=0.5, dstate_std=0.5),
    # hidden sizes that take the split-K step kernels (H >= 1024, multiple of 64)
    Config("sk1", L=2, T=3, B=5, I=40, H=1024, state_std=0.5, dstate_std=0.5),
    Config("sk2", L=2, T=2, B=70, I=24, H=1088, state_std=0.5, dstate_std=0.5),
]


# (hidden sizes from 512 on are never padded: they have one variant)
ODD_CASES = [(c, f, nopad) for f in (0, 1, 3, 4, 5) for c in ODD for nopad in (False, True) if not (nopad and c.H >= 512)]


@pytest.mark.parametrize("cfg,flags,nopad", ODD_CASES,
                         ids=[f"{'as_given' if n else 'padded'}-{c.name}-{f}" for c, f, n in ODD_CASES])
def test_odd_shapes(cfg, flags, nopad, knobs):
    if nopad:
        knobs(LSTM_NO_PAD="1")
    run_case(cfg, 3, flags)


# The forward step kernel with 4, 8 and 16 hidden units per workgroup (the automatic choice depends on the hidden
# size: 16 only from H = 3200 on), ragged shapes as given; B = 50 takes the variants built for two waves per SIMD.
STEPK = [ODD[2], ODD[4], ODD[6],
         Config("odd6", L=1, T=3, B=50, I=20, H=72, state_std=0.5, dstate_std=0.5),
         Config("sk3", L=1, T=2, B=50, I=24, H=1024, state_std=0.5, dstate_std=0.5)]


@pytest.mark.parametrize("mt", ["1", "2", "4"])
@pytest.mark.parametrize("cfg", STEPK, ids=[c.name for c in STEPK])
def test_step_kernel_units_per_workgroup(cfg, mt, knobs):
    _, binding, _ = _mods()
    knobs(LSTM_NO_PAD="1")
    knobs(LSTM_STEP_MT=mt)
    run_case(cfg, 19, binding.LSTM_PATH_STEP)


# ------------------------------------------------------------------ hidden sizes padded to the persistent kernels'
PADDED = [
    Config("h384", L=2, T=5, B=20, I=384, H=384, state_std=0.3, dstate_std=0.3),      # I == H before padding, not after
    Config("h200", L=3, T=4, B=64, I=100, H=200, state_std=0.3, dstate_std=0.3),
    Config("h72", L=1, T=40, B=33, I=72, H=72, state_std=0.3, dstate_std=0.3),
    Config("h300b130", L=2, T=3, B=130, I=40, H=300, state_std=0.3, dstate_std=0.3),  # three batch slices
    Config("h511", L=5, T=3, B=7, I=511, H=511, state_std=0.3, dstate_std=0.3),       # odd size, two groups of layers
    Config("h800", L=2, T=3, B=40, I=800, H=800, state_std=0.3, dstate_std=0.3),      # to 1024: the one-layer kernels
    Config("h560", L=1, T=32, B=9, I=48, H=560, state_std=0.3, dstate_std=0.3),       # just above 512, few rows: to 1024 as well
    Config("h1500", L=2, T=3, B=20, I=64, H=1500, state_std=0.3, dstate_std=0.3),     # to 2048 (few rows only)
]


@pytest.mark.parametrize("cfg", PADDED, ids=[c.name for c in PADDED])
@pytest.mark.parametrize("with_states", [True, False])
def test_padded_hidden_sizes(cfg, with_states):
    torch, binding, _ = _mods()
    assert binding.lstm_auto_path(*cfg.dims, 0) == binding.LSTM_PATH_PERSISTENT
    assert binding.lstm_auto_path(*cfg.dims, 1) == binding.LSTM_PATH_PERSISTENT
    r, ref = run_case(cfg, 17, 0, with_states=with_states, with_dstates=with_states)
    y_train = r.y.clone()
    r.y.fill_(float("nan"))
    binding.check(r.forward(flags=0, inference=True))
    torch.cuda.synchronize()
    assert torch.equal(r.y, y_train)


# The smallest networks: one workgroup runs a whole pass (H = 8, 16, 32; few rows, few layers).
MICRO = [
    Config("m8", L=2, T=5, B=3, I=5, H=8, state_std=0.5, dstate_std=0.5),
    Config("m16", L=3, T=7, B=8, I=64, H=16, state_std=0.5, dstate_std=0.5),
    Config("m32", L=4, T=9, B=8, I=32, H=32, state_std=0.5, dstate_std=0.5),
    Config("m32b2", L=2, T=6, B=2, I=64, H=32, state_std=0.5, dstate_std=0.5),
    Config("m32b1", L=1, T=40, B=1, I=20, H=32, state_std=0.5, dstate_std=0.5),
    Config("m32T1", L=2, T=1, B=7, I=1, H=32, state_std=0.5, dstate_std=0.5),
    # more steps than are staged in LDS at a time: two lots forward, six backward; with inputs of 5 floats (no
    # 16-byte alignment: the scalar staging loop) two forward and nine backward
    Config("m32long", L=2, T=60, B=8, I=64, H=32, state_std=0.5, dstate_std=0.5),
    Config("m8long", L=1, T=400, B=8, I=5, H=8, state_std=0.5, dstate_std=0.5),
]


@pytest.mark.parametrize("cfg", MICRO, ids=[c.name for c in MICRO])
@pytest.mark.parametrize("with_states", [True, False])
def test_one_workgroup_per_pass(cfg, with_states, knobs):
    _, binding, _ = _mods()
    knobs(LSTM_MICRO="2")  # every shape the kernels take, not only those where they are the automatic choice
    assert binding.lstm_auto_path(*cfg.dims, 0) == binding.LSTM_PATH_STEP
    assert binding.lstm_auto_path(*cfg.dims, 1) == binding.LSTM_PATH_STEP
    run_case(cfg, 11, 0, with_states=with_states, with_dstates=with_states)
    run_case(cfg, 12, binding.LSTM_PATH_STEP, with_states=with_states, with_dstates=with_states)


# ------------------------------------------------------------------ optional pointers, inference
@pytest.mark.parametrize("hidden", [24, 32], ids=["h24", "h32_one_workgroup"])
@pytest.mark.parametrize("nopad", [False, True], ids=["padded", "as_given"])
def test_null_optionals_and_inference(nopad, hidden, knobs):
    torch, binding, runner = _mods()
    if nopad:
        knobs(LSTM_NO_PAD="1")
    if hidden == 32:
        knobs(LSTM_MICRO="2")
    cfg = Config("opt", L=2, T=4, B=6, I=16, H=hidden)
    for flags in (0, 4):
        d, ref = oracle_results(cfg, 5, with_states=False, with_dstates=False)
        r = runner.LstmRunner(cfg.dims, d, with_states=False, with_dstates=False)
        r.poison()
        binding.check(r.forward(flags=flags, want_states=False))
        binding.check(r.backward(flags=flags, want_dx=False, want_dstates=False))
        torch.cuda.synchronize()
        assert_close(r.fwd_outputs(), ref, ("y",), FWD_TOL)
        assert_close(r.bwd_outputs(), ref, ("dW", "dR", "db"), BWD_TOL)
        assert torch.isnan(r.hT).all() and torch.isnan(r.dx).all() and torch.isnan(r.dh0).all()
        y_train = r.y.clone()
        r.y.fill_(float("nan"))
        binding.check(r.forward(flags=flags, inference=True))
        torch.cuda.synchronize()
        assert torch.equal(r.y, y_train)


def test_large_minibatch_takes_the_gemm_rung_forward():
    """Once one step's [B x 4H] x [H] product fills every CU with 128 x 128 tiles the automatic forward path is the
    grouped-GEMM + fused point-wise rung, the backward path stays the step kernel; the two must work together."""
    _, binding, _ = _mods()
    cfg = Config("bigB", L=2, T=2, B=512, I=64, H=2048, state_std=0.3, dstate_std=0.3)
    assert binding.lstm_auto_path(*cfg.dims, 0) == binding.LSTM_PATH_FUSED
    assert binding.lstm_auto_path(*cfg.dims, 1) in (binding.LSTM_PATH_STEP, binding.LSTM_PATH_WAVEFRONT)
    run_case(cfg, 13, 0)


# ------------------------------------------------------------------ the large end of the hidden-size / minibatch sweep
# Section 3.2 sweeps hidden sizes up to 4096 and minibatches up to 256; these are the kernels that the sweep times
# there, compared with the oracle on two or three steps: the forward step kernel with 16 units per workgroup and the
# split-K backward kernel (H = 4096), the grouped-GEMM rung that the automatic forward path takes once one step fills
# the chip (B = 256), and the step kernels at H = 2048 with 256 rows (two waves per SIMD).
SWEEP_END = [
    (Config("s4096b32", L=1, T=2, B=32, I=64, H=4096, state_std=0.3, dstate_std=0.3), 0),
    (Config("s4096L2b64", L=2, T=2, B=64, I=4096, H=4096, state_std=0.3, dstate_std=0.3), 0),
    (Config("s4096b256", L=1, T=2, B=256, I=64, H=4096, state_std=0.3, dstate_std=0.3), 0),
    (Config("s2048b256", L=2, T=2, B=256, I=128, H=2048, state_std=0.3, dstate_std=0.3), 4),
]
SWEEP_END += [(Config("s4096L2b32", L=2, T=3, B=32, I=64, H=4096, state_std=0.3, dstate_std=0.3), f) for f in (3, 4, 5)]
SWEEP_END += [(Config("s4096b256", L=1, T=2, B=256, I=64, H=4096, state_std=0.3, dstate_std=0.3), f) for f in (3, 4, 5)]
SWEEP_END += [(Config("s2048L1b256", L=1, T=3, B=256, I=64, H=2048, state_std=0.3, dstate_std=0.3), f) for f in (0, 3, 4, 5)]


@pytest.mark.parametrize("cfg,flags", SWEEP_END, ids=[f"{c.name}-path{f}" for c, f in SWEEP_END])
def test_large_end_of_the_sweep(cfg, flags):
    run_case(cfg, 29, flags)


# ------------------------------------------------------------------ determinism (doubles as a race detector)
@pytest.mark.parametrize("name", ["cfg1", "cfg3", "cfg4", "cfg5"])
def test_bitwise_repeatable(name):
    torch, binding, runner = _mods()
    cfg = CONFIGS[name]
    d = make_inputs(cfg, 0)
    r = runner.LstmRunner(cfg.dims, d)
    outs = []
    for it in range(3):
        r.poison()
        binding.check(r.forward())
        binding.check(r.backward())
        torch.cuda.synchronize()
        outs.append({k: getattr(r, k).clone() for k in FWD + BWD})
    for k in FWD + BWD:
        assert torch.equal(outs[0][k], outs[1][k]) and torch.equal(outs[0][k], outs[2][k]), k


@pytest.mark.parametrize("launch", ["unchained", "chained", "cooperative"])
@pytest.mark.parametrize("dims", [(4, 100, 16, 256), (8, 60, 32, 256)], ids=["b16", "b32"])
def test_two_streams_sharing_the_cus_do_not_disturb_each_other(dims, launch, knobs):
    """Two calls on two streams: each must give exactly what it gives alone.  Unchained ordinary launches let the two
    persistent kernels run on the same CUs at once where both fit (small register footprint): this caught a 16-byte
    write-through store issued from inline assembly without the idle cycles a wide store needs before its data
    registers are overwritten.  The default chains the persistent launches of the process; cooperative launches are
    the third mode."""
    torch, binding, runner = _mods()
    if launch != "chained":
        knobs(**{"LSTM_PLAIN_LAUNCH" if launch == "unchained" else "LSTM_COOP_LAUNCH": "1"})
    L, T, B, H = dims
    cfg = Config("two", L=L, T=T, B=B, I=H, H=H, state_std=0.1)
    r1, r2 = runner.LstmRunner(cfg.dims, make_inputs(cfg, 1)), runner.LstmRunner(cfg.dims, make_inputs(cfg, 2))
    alone = []
    for r in (r1, r2):
        binding.check(r.forward())
        binding.check(r.backward())
        torch.cuda.synchronize()
        alone.append({k: getattr(r, k).clone() for k in FWD + BWD})
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for trial in range(4):
        for first_bwd in (False, True):
            with torch.cuda.stream(s1):
                binding.check(r1.backward() if first_bwd else r1.forward())
            with torch.cuda.stream(s2):
                binding.check(r2.backward())
            with torch.cuda.stream(s1):
                binding.check(r1.backward())
            torch.cuda.synchronize()
            for r, ref in ((r1, alone[0]), (r2, alone[1])):
                for k in FWD + BWD:
                    assert torch.equal(getattr(r, k), ref[k]), (trial, first_bwd, k)


# ------------------------------------------------------------------ boundary identity on the GPU
@pytest.mark.parametrize("nopad", [False, True], ids=["padded", "as_given"])
def test_split_T_chaining_on_gpu(nopad, knobs):
    torch, binding, runner = _mods()
    if nopad:
        knobs(LSTM_NO_PAD="1")
    cfg = Config("chain", L=2, T=8, B=16, I=32, H=64, state_std=0.3)
    d = make_inputs(cfg, 7)
    full = runner.LstmRunner(cfg.dims, d)
    binding.check(full.forward())
    T1 = 3
    d1 = dict(d, x=d["x"][:T1], dy=d["dy"][:T1])
    r1 = runner.LstmRunner((cfg.L, T1, cfg.B, cfg.I, cfg.H), d1)
    binding.check(r1.forward())
    torch.cuda.synchronize()
    d2 = dict(d, x=d["x"][T1:], dy=d["dy"][T1:], h0=r1.hT.cpu().numpy(), c0=r1.cT.cpu().numpy())
    r2 = runner.LstmRunner((cfg.L, cfg.T - T1, cfg.B, cfg.I, cfg.H), d2)
    binding.check(r2.forward())
    torch.cuda.synchronize()
    y12 = torch.cat([r1.y, r2.y])
    assert float((y12 - full.y).abs().max()) < 1e-5
    assert float((r2.hT - full.hT).abs().max()) < 1e-5


# ------------------------------------------------------------------ chunk length of the stream wavefront
@pytest.mark.parametrize("chunks", [1, 2, 3, 7, 100])
def test_wavefront_chunk_counts(chunks):
    """Section 2.3's s (steps per batched input product) is a per-shape setting of the wavefront path: any count gives
    the same results."""
    _, binding, _ = _mods()
    cfg = Config("chunks", L=3, T=7, B=20, I=48, H=640, state_std=0.3, dstate_std=0.3)
    try:
        binding.check(binding.lstm_set_wavefront_chunks(*cfg.dims, chunks))
        run_case(cfg, 23, binding.LSTM_PATH_WAVEFRONT)
    finally:
        binding.lstm_set_wavefront_chunks(*cfg.dims, 0)


# ------------------------------------------------------------------ autotuner
def test_autotune_pins_a_path_and_results_stay_right():
    _, binding, _ = _mods()
    from paper_1604_01946_amd import autotune
    cfg = Config("tune", L=2, T=6, B=40, I=128, H=128, state_std=0.3, dstate_std=0.3)
    try:
        r = autotune.tune(*cfg.dims, iters=2)
        assert set(r["forward"]) >= {"step", "wavefront"} and set(r["backward"]) >= {"step", "wavefront"}
        names = {v: k for k, v in binding.PATH_NAMES.items()}
        assert binding.lstm_auto_path(*cfg.dims, 0) == names[r["best"][0]]
        assert binding.lstm_auto_path(*cfg.dims, 1) == names[r["best"][1]]
        assert r["best_chunks"] in ("default", 1, 2, 4) and set(r["wavefront_chunks"]) == {"default", 1, 2, 4}
        run_case(cfg, 5, 0)
        run_case(cfg, 5, binding.LSTM_PATH_WAVEFRONT)   # with the chunk count the tuner pinned
    finally:
        binding.lstm_set_path(*cfg.dims, 0, binding.LSTM_PATH_AUTO)
        binding.lstm_set_path(*cfg.dims, 1, binding.LSTM_PATH_AUTO)
        binding.lstm_set_wavefront_chunks(*cfg.dims, 0)
