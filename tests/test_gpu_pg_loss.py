"""GPU parity of the clipped policy-gradient loss (fused LM-head form and
logits-in form, forward and backward) against the fp64 oracle, through the C ABI.

Tolerances: lse / logp absolute 2e-4 (bf16 inputs, fp32 accumulation), loss 2e-3
relative, gradients 1e-2 relative L2; fp32 inputs: lse / logp absolute 2e-5."""
import numpy as np
import pytest
import torch

from paper_2509_13232_amd import workloads as wl
from pg_cases import Case, check_forward, f64, rel_l2, say

pytestmark = pytest.mark.gpu
GRAD_TOL = 1e-2


@pytest.fixture(scope="module")
def spo():
    from paper_2509_13232_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


MID = wl.scaled(wl.CONFIGS["C2"], name="mid", H=256, V=3000, mask_span=(4, 40))
MID_LENGTHS = [37, 300, 1, 255, 120]  # T = 713: three token tiles, ragged tail; V: 11 tiles + 184


@pytest.fixture(params=[False, True], ids=["fwd_then_bwd", "one_call"])
def one_call(request):
    """The two ways to the gradients: spo_pg_loss_fwd followed by spo_pg_loss_bwd (the logits are
    formed twice), or spo_pg_loss_fwd_bwd (formed once and kept, piece by piece, as fp16)."""
    return request.param


def run_fwd_bwd(spo, case, w_layout=0, chunk_tokens=0, dx_dtype=torch.float32, dw_dtype=torch.float32,
                one_call=False):
    desc = case.to_gpu(spo, w_layout)
    if one_call:
        *fwd, dx, dw = spo.spo_pg_loss_fwd_bwd(desc, 1.0, d_hidden_dtype=dx_dtype, d_W_dtype=dw_dtype,
                                               chunk_tokens=chunk_tokens)
        fwd = tuple(fwd)
    else:
        fwd = spo.spo_pg_loss_fwd(desc)
        dx, dw = spo.spo_pg_loss_bwd(desc, fwd[1], fwd[2], 1.0, d_hidden_dtype=dx_dtype, d_W_dtype=dw_dtype,
                                     chunk_tokens=chunk_tokens)
    torch.cuda.synchronize()
    if w_layout == 1:
        dw = dw.t()
    return fwd, dx, dw


@pytest.mark.parametrize("w_layout", [0, 1])
def test_tiny_spo_step_fp32(spo, oracle, w_layout, one_call):
    cfg = wl.CONFIGS["C1"]
    say(f"fused fp32 C1 T=512 H=128 V=1000 w_layout={w_layout} one_call={one_call}")
    case = Case(cfg)
    assert case.T == 512
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, w_layout=w_layout, one_call=one_call)
    check_forward(case, oracle, fwd, atol_logp=2e-5)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL
    assert rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL


@pytest.mark.parametrize("w_layout", [0, 1])
@pytest.mark.parametrize("w_scale,mask_frac", [(1.0, 0.0), (1.0, 0.25), (30.0, 0.25)])
def test_fused_bf16_matches_oracle(spo, oracle, w_layout, w_scale, mask_frac, one_call):
    say(f"fused bf16 mid T=713 H=256 V=3000 w_layout={w_layout} w_scale={w_scale} mask={mask_frac} one_call={one_call}")
    case = Case(MID, MID_LENGTHS, w_scale=w_scale, mask_frac=mask_frac)
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, w_layout, one_call=one_call)
    ref = check_forward(case, oracle, fwd)
    assert 0 < ref["active"].sum() < case.T          # both branches of the min occur
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL
    assert rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
    # the softmax part alone (gradient minus the rank-one target term), which a flat
    # softmax hides inside the total: bounded by the bf16 rounding of the logit
    # gradients of both parts
    g = rb["g"]
    Wd, Hd = f64(case.W), f64(case.hidden)
    onehot_dx = g[:, None] * Wd[case.target]
    soft_ref = rb["d_hidden"] - onehot_dx
    soft_gpu = f64(dx) - onehot_dx
    # (a target entry of dZ is rounded to bf16 once: at most 2^-9 of it)
    bound = GRAD_TOL * np.linalg.norm(soft_ref) + 1.1 * 2.0 ** -9 * np.linalg.norm(onehot_dx)
    assert np.linalg.norm(soft_gpu - soft_ref) <= bound
    if w_scale > 1.0:   # peaked softmax: the softmax part is as large as the target part
        assert np.linalg.norm(soft_ref) > 0.3 * np.linalg.norm(onehot_dx)
        assert rel_l2(soft_gpu, soft_ref) < 2 * GRAD_TOL
    # rows of masked tokens are exactly zero; softmax rows sum to one
    if case.mask is not None:
        assert not dx[torch.as_tensor(case.mask == 0)].any()
    col = f64(dw).sum(axis=0)
    assert np.abs(col).max() <= 2e-2 * np.abs(f64(dw)).sum(axis=0).max()
    del Hd


def test_backward_chunks_and_output_dtypes(spo, oracle, one_call):
    say(f"fused bf16 mid, chunk_tokens=256 (3 chunks), bf16 outputs, one_call={one_call}")
    case = Case(MID, MID_LENGTHS, mask_frac=0.25)
    case.set_old_from_oracle(oracle)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    f1, dx1, dw1 = run_fwd_bwd(spo, case, chunk_tokens=256, one_call=one_call)
    f2, dx2, dw2 = run_fwd_bwd(spo, case, chunk_tokens=0, one_call=one_call)
    check_forward(case, oracle, f1)
    assert torch.allclose(f1[1], f2[1], atol=1e-5, rtol=0)            # a token's log-prob does not depend on the pieces
    assert rel_l2(f64(dx1), rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw1), rb["d_W"]) < GRAD_TOL
    assert rel_l2(f64(dx1), f64(dx2)) < 1e-5           # rows depend on the chunking only through the order of fp32 sums
    assert rel_l2(f64(dw1), f64(dw2)) < 1e-5           # fp32 partial sums in another order
    _, dx3, dw3 = run_fwd_bwd(spo, case, chunk_tokens=512, dx_dtype=torch.bfloat16, dw_dtype=torch.bfloat16,
                              one_call=one_call)
    assert dx3.dtype == torch.bfloat16 and dw3.dtype == torch.bfloat16
    assert rel_l2(f64(dx3), rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw3), rb["d_W"]) < GRAD_TOL


@pytest.mark.parametrize("mask_frac", [None, 0.25], ids=["no_mask", "masked"])
def test_one_call_with_only_one_of_the_two_gradients(spo, oracle, mask_frac):
    # d_hidden alone, d_W alone, neither (loss and log-probs only): the one call skips what is not asked for
    say(f"one call, single outputs, mask={mask_frac}")
    case = Case(MID, MID_LENGTHS, mask_frac=mask_frac)
    case.set_old_from_oracle(oracle)
    desc = case.to_gpu(spo)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    *fwd, dx, dw = spo.spo_pg_loss_fwd_bwd(desc, 1.0, d_hidden_dtype=torch.float32, want_d_W=False)
    torch.cuda.synchronize()
    check_forward(case, oracle, tuple(fwd))
    assert dw is None and rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL
    *fwd, dx, dw = spo.spo_pg_loss_fwd_bwd(desc, 1.0, want_d_hidden=False)
    torch.cuda.synchronize()
    check_forward(case, oracle, tuple(fwd))
    assert dx is None and rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
    *fwd, dx, dw = spo.spo_pg_loss_fwd_bwd(desc, 1.0, want_d_hidden=False, want_d_W=False)
    torch.cuda.synchronize()
    check_forward(case, oracle, tuple(fwd))
    assert dx is None and dw is None
    # grad_loss scales both gradients
    _, _, _, _, dx2, dw2 = spo.spo_pg_loss_fwd_bwd(desc, -2.5, d_hidden_dtype=torch.float32)
    torch.cuda.synchronize()
    assert rel_l2(f64(dx2), -2.5 * rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw2), -2.5 * rb["d_W"]) < GRAD_TOL


@pytest.mark.parametrize("w_layout", [0, 1])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_head_gradient_on_ragged_shapes(spo, oracle, w_layout, dtype, one_call):
    # dW contracts over tokens from rows of dZ and of the hidden states: a vocabulary that is
    # neither a multiple of the tile nor of the 8-element pieces the rows are fetched in, a
    # hidden size below one tile, a token count with a ragged last tile.  Element-wise check:
    # a misplaced column or a piece fetched past the end of a row shows up in single entries.
    say(f"fused {dtype} ragged T=300 H=192 V=1003 w_layout={w_layout} one_call={one_call}")
    cfg = wl.scaled(MID, name="ragged", H=192, V=1003, dtype=dtype)
    case = Case(cfg, [130, 170])
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, w_layout, one_call=one_call)
    check_forward(case, oracle, fwd, atol_logp=2e-4 if dtype == "bf16" else 2e-5)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    assert dw.shape == (1003, 192)
    assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
    scale = np.abs(rb["d_W"]).max()
    np.testing.assert_allclose(f64(dw), rb["d_W"], atol=2e-2 * scale, rtol=0)
    # every vocabulary row's gradient against its own size (the target rows dominate the total)
    rows = np.linalg.norm(f64(dw) - rb["d_W"], axis=1)
    assert (rows <= 5e-2 * np.linalg.norm(rb["d_W"], axis=1) + 1e-3 * scale).all()


@pytest.mark.parametrize("lengths,V,H,w_layout,chunk", [
    ([1], 5, 64, 0, 0),              # one token, vocabulary below one fetch piece
    ([1], 5, 64, 1, 0),
    ([200, 55], 63, 128, 1, 0),      # one short of a k-block of the vocabulary, one short of a token tile
    ([129, 128], 65, 64, 0, 256),    # one past both, two chunks
    ([500, 12], 1023, 192, 1, 256),  # one short of four vocabulary tiles
    ([150, 150], 2049, 256, 0, 0),   # one past eight vocabulary tiles
    ([40], 300, 320, 1, 0),          # hidden size between one and two tiles
])
def test_corner_shapes_match_oracle(spo, oracle, lengths, V, H, w_layout, chunk, one_call):
    # sizes that sit on, just below and just above the tile, block and fetch-piece boundaries of
    # the contraction kernels, forward and both gradients against the oracle
    say(f"fused bf16 corner T={sum(lengths)} H={H} V={V} w_layout={w_layout} chunk={chunk} one_call={one_call}")
    cfg = wl.scaled(MID, name="corner", H=H, V=V)
    case = Case(cfg, lengths)
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, w_layout, chunk_tokens=chunk, one_call=one_call)
    check_forward(case, oracle, fwd)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    assert dw.shape == (V, H) and dx.shape == (sum(lengths), H)
    if np.any(rb["d_hidden"]):
        assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
        scale = np.abs(rb["d_W"]).max()
        np.testing.assert_allclose(f64(dw), rb["d_W"], atol=2e-2 * scale, rtol=0)
    else:   # every token ended on the clipped branch
        assert not dx.any() and not dw.any()


@pytest.mark.parametrize("w_layout,chunk", [(0, 0), (1, 512)])
def test_last_round_of_dW_tiles_cut_along_the_tokens(spo, oracle, w_layout, chunk, one_call):
    # 33 x 8 = 264 tiles of d_W on 256 compute units: the 8 tiles of the last round are launched on
    # their own, each cut into 8 runs of tokens whose partial tiles are added in order (with chunk =
    # 512 two launches add into d_W; 900 tokens are 16 k-steps: two per part in the first chunk, one or
    # none in the second).  Every entry against the oracle, the tiles of the last round on their own.
    V, H = 8200, 2048
    say(f"fused bf16 T=900 H={H} V={V} w_layout={w_layout} chunk={chunk} one_call={one_call}: d_W tail tiles")
    cfg = wl.scaled(MID, name="tail", H=H, V=V)
    case = Case(cfg, [400, 500])
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, w_layout, chunk_tokens=chunk, one_call=one_call)
    check_forward(case, oracle, fwd)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    got = f64(dw)
    assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL and rel_l2(got, rb["d_W"]) < GRAD_TOL
    scale = np.abs(rb["d_W"]).max()
    np.testing.assert_allclose(got, rb["d_W"], atol=2e-2 * scale, rtol=0)
    # in the row-major order of 256 x 256 tiles of the kernel's output ([V, H], or [H, V] for w_layout 1)
    # the last 8 tiles are the last tile row: vocabulary entries from 8192 on, or hidden units from 1792 on
    tail = (slice(8192, V), slice(None)) if w_layout == 0 else (slice(None), slice(1792, H))
    assert np.abs(rb["d_W"][tail]).max() > 0
    assert rel_l2(got[tail], rb["d_W"][tail]) < 2 * GRAD_TOL


@pytest.mark.parametrize("mask_frac", [None, 0.02], ids=["no_mask", "masked"])
def test_last_round_of_dHidden_tiles_cut_along_the_vocabulary(spo, oracle, mask_frac, one_call):
    # ~8300 rows x 2048 hidden units: 33 x 8 = 264 tiles of d_hidden on 256 compute units, so the 8 tiles
    # of the last round (the last 52 tokens) are cut into 8 runs of the vocabulary (9 k-steps: five parts
    # have work).  Without a mask the one call knows the tile count on the host; otherwise the number of
    # active tokens, and with it whether and where to cut, is known on the device only.
    # (token counts chosen so that the rows the contraction runs over, all tokens or the ~97-99 % with a
    # gradient, fall into the 33rd row tile)
    T = 8300 if (one_call and mask_frac is None) else 8400 if mask_frac is None else 8560
    say(f"fused bf16 T={T} H=2048 V=520 mask={mask_frac} one_call={one_call}: d_hidden tail tiles")
    cfg = wl.scaled(MID, name="dxtail", H=2048, V=520)
    case = Case(cfg, [4000, T - 4000], mask_frac=mask_frac)
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, one_call=one_call)
    ref = check_forward(case, oracle, fwd)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    n_active = int(np.count_nonzero(rb["g"]))
    rows = T if (one_call and mask_frac is None) else n_active
    assert 8192 < rows <= 8448, rows        # 33 row tiles: a last round of 8 tiles
    got = f64(dx)
    assert rel_l2(got, rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
    per_row = np.linalg.norm(got - rb["d_hidden"], axis=1)
    scale = np.linalg.norm(rb["d_hidden"], axis=1)
    assert (per_row <= 2 * GRAD_TOL * scale + 1e-12).all()     # every token's row, those of the cut tiles included
    assert not got[scale == 0].any()


DEEP = wl.scaled(wl.CONFIGS["C2"], name="deep", H=320, V=1100)
DEEP_LENGTHS = [9000, 7000, 12001, 5000, 6999]  # T = 40000: 157 token tiles, three chunks of 16384


@pytest.mark.timeout(600)
@pytest.mark.parametrize("w_layout,w_scale", [(0, 1.0), (1, 1.0), (0, 30.0)])
def test_dense_deep_token_contraction_of_dW(spo, oracle, w_layout, w_scale, one_call):
    # The head gradient contracts over tokens.  Here nothing is masked, so every chunk of 16384
    # tokens is one launch with 256 steps of the contraction, and the three chunks add into the
    # same fp32 d_W (read-modify-write across launches), as in the benchmark configuration.
    # Every entry of d_W and d_hidden is compared with the oracle; the softmax part of d_W
    # (d_W minus the rank-one terms of the sampled tokens) is compared on its own, because with
    # flat logits it hides inside the total; w_scale = 30 makes it as large as the target part.
    say(f"fused bf16 deep T=40000 H=320 V=1100 chunk=16384 w_layout={w_layout} w_scale={w_scale} one_call={one_call}")
    case = Case(DEEP, DEEP_LENGTHS, w_scale=w_scale)
    assert case.T == 40000 and case.mask is None
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, w_layout, chunk_tokens=16384, one_call=one_call)
    ref = check_forward(case, oracle, fwd)
    assert ref["active"].sum() > 2 * 16384                   # three chunks of active tokens
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    got_dw, got_dx = f64(dw), f64(dx)
    assert rel_l2(got_dx, rb["d_hidden"]) < GRAD_TOL and rel_l2(got_dw, rb["d_W"]) < GRAD_TOL
    scale = np.abs(rb["d_W"]).max()
    np.testing.assert_allclose(got_dw, rb["d_W"], atol=2e-2 * scale, rtol=0)
    rows = np.linalg.norm(got_dw - rb["d_W"], axis=1)        # no vocabulary row hides in the norm
    assert (rows <= 2 * GRAD_TOL * np.linalg.norm(rb["d_W"], axis=1) + 1e-3 * scale).all()
    # softmax part: subtract sum over the tokens that sampled v of g_t h_t
    g, Hd = rb["g"], f64(case.hidden)
    onehot_dw = np.zeros_like(rb["d_W"])
    np.add.at(onehot_dw, case.target, g[:, None] * Hd)
    soft_ref, soft_gpu = rb["d_W"] - onehot_dw, got_dw - onehot_dw
    # bf16 rounding of a target entry of dZ is at most 2^-9 of it, independently per token
    bound = GRAD_TOL * np.linalg.norm(soft_ref) + 1.1 * 2.0 ** -9 * np.linalg.norm(onehot_dw)
    assert np.linalg.norm(soft_gpu - soft_ref) <= bound
    if w_scale > 1.0:
        assert np.linalg.norm(soft_ref) > 0.3 * np.linalg.norm(onehot_dw)
        assert rel_l2(soft_gpu, soft_ref) < 2 * GRAD_TOL
    # the same gradients from one chunk that holds every token: only the order of the fp32 sums differs
    # (of dW over the chunks, of dHidden over the parts a small chunk's vocabulary contraction is cut into)
    _, dx1, dw1 = run_fwd_bwd(spo, case, w_layout, chunk_tokens=0, one_call=one_call)
    assert rel_l2(f64(dx1), got_dx) < 1e-5 and rel_l2(f64(dw1), got_dw) < 1e-4
    _, dx2, dw2 = run_fwd_bwd(spo, case, w_layout, chunk_tokens=16384, one_call=one_call)
    assert torch.equal(dx2, dx) and torch.equal(dw2, dw if w_layout == 0 else dw)   # same call, same bits


@pytest.mark.parametrize("keep,chunk", [(256, 256), (257, 256), (1, 0), (300, 512), (511, 256)])
def test_backward_runs_over_active_tokens_only(spo, oracle, keep, chunk, one_call):
    # A sparse loss mask: the backward gathers the tokens that carry a gradient and works on
    # that list, `keep` of them here, chosen to end exactly on, one past, and far from the
    # boundaries of token tiles and chunks.  Rows of all other tokens must be exact zeros.
    say(f"fused bf16 mid, {keep} unmasked tokens, chunk_tokens={chunk} one_call={one_call}")
    case = Case(MID, MID_LENGTHS)
    case.set_old_from_oracle(oracle)
    rng = np.random.default_rng(keep)
    live = np.sort(rng.choice(case.T, keep, replace=False))
    case.mask = np.zeros(case.T, np.uint8)
    case.mask[live] = 1
    fwd, dx, dw = run_fwd_bwd(spo, case, chunk_tokens=chunk, one_call=one_call)
    check_forward(case, oracle, fwd)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
    dead = np.setdiff1d(np.arange(case.T), live)
    assert not dx[torch.as_tensor(dead, device="cuda")].any()
    # a clipped token is dropped from the list like a masked one
    zero_rows = np.flatnonzero(~rb["d_hidden"].any(axis=1))
    assert not dx[torch.as_tensor(zero_rows, device="cuda")].any()


def test_cu_seqlens_may_start_anywhere(spo, oracle):
    # a mini-batch cut out of a packed batch keeps the batch's offsets: only differences count
    say("fused bf16 mid, cu_seqlens shifted by a constant")
    case = Case(MID, MID_LENGTHS, mask_frac=0.25)
    case.set_old_from_oracle(oracle)
    a = run_fwd_bwd(spo, case)
    case.cu = (case.cu.astype(np.int64) + 123456).astype(np.int32)
    b = run_fwd_bwd(spo, case)
    assert torch.equal(a[0][0], b[0][0]) and torch.equal(a[0][1], b[0][1])
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


def test_results_are_bitwise_reproducible(spo, oracle, one_call):
    say(f"fused bf16 mid, determinism, one_call={one_call}")
    case = Case(MID, MID_LENGTHS)
    case.set_old_from_oracle(oracle)
    a = run_fwd_bwd(spo, case, chunk_tokens=256, one_call=one_call)
    b = run_fwd_bwd(spo, case, chunk_tokens=256, one_call=one_call)
    assert torch.equal(a[0][0], b[0][0]) and torch.equal(a[0][1], b[0][1])
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


def test_mini_batches_accumulate_into_dW(spo, oracle, one_call):
    # two mini-batches of whole responses, the batch-wide normalised advantages,
    # gradients accumulated into one d_W (one optimiser step per mini-batch is the
    # caller's business; the kernel only has to add)
    say(f"fused bf16 mid, two mini-batches, accumulate_dW, one_call={one_call}")
    case = Case(MID, MID_LENGTHS)
    case.set_old_from_oracle(oracle)
    h, w, tg, old, mk, ad, cu = case.oracle_inputs()
    d = "cuda"
    hidden, W = case.hidden.to(d), case.W.to(d)
    target = torch.as_tensor(case.target).to(d)
    oldg = torch.as_tensor(case.old).to(d)
    adv = torch.as_tensor(case.adv).to(d)
    cug = torch.as_tensor(case.cu).to(d)
    dW = torch.zeros_like(W, dtype=torch.float32)
    ref_dw = np.zeros_like(w)
    for (b0, b1) in ((0, 2), (2, 5)):
        t0, t1 = int(cu[b0]), int(cu[b1])
        desc = spo.make_desc(hidden[t0:t1], W, target[t0:t1], oldg[t0:t1], None, adv[b0:b1],
                             cug[b0:b1 + 1], *case.eps)
        if one_call:
            loss, _, _, _, dx, _ = spo.spo_pg_loss_fwd_bwd(desc, 1.0, d_hidden_dtype=torch.float32, d_W=dW,
                                                           accumulate_dW=True)
        else:
            loss, logp, lse, _ = spo.spo_pg_loss_fwd(desc)
            dx, _ = spo.spo_pg_loss_bwd(desc, logp, lse, 1.0, d_hidden_dtype=torch.float32, d_W=dW,
                                        accumulate_dW=True)
        torch.cuda.synchronize()
        sub_cu = (cu[b0:b1 + 1] - cu[b0]).astype(np.int32)
        rf = oracle.pg_loss_fwd(h[t0:t1], w, tg[t0:t1], old[t0:t1], None, ad[b0:b1], sub_cu, *case.eps)
        rb = oracle.pg_loss_bwd(h[t0:t1], w, tg[t0:t1], old[t0:t1], None, ad[b0:b1], sub_cu, *case.eps)
        assert abs(loss.item() - rf["loss"]) <= 2e-3 * abs(rf["loss"]) + 1e-7
        assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL
        ref_dw += rb["d_W"]
    assert rel_l2(f64(dW), ref_dw) < GRAD_TOL


def test_degenerate_inputs(spo, oracle, one_call):
    say(f"fused: all tokens masked, one_call={one_call}")
    case = Case(MID, [40, 60], mask_frac=0.5)
    case.set_old_from_oracle(oracle)
    case.mask = np.zeros(case.T, np.uint8)
    fwd, dx, dw = run_fwd_bwd(spo, case, one_call=one_call)
    assert fwd[0].item() == 0.0 and not dx.any() and not dw.any()
    ref = oracle.pg_loss_fwd(*case.oracle_inputs(), *case.eps)
    np.testing.assert_allclose(f64(fwd[1]), ref["logp"], atol=2e-4)     # log-probs are still produced
    say("fused: one token, vocabulary smaller than a tile")
    tiny = wl.scaled(MID, name="tiny", H=64, V=100)
    case = Case(tiny, [1], adv=[1.5])
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, one_call=one_call)
    check_forward(case, oracle, fwd)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
    say("fused: empty responses inside the batch")
    case = Case(MID, [0, 70, 0, 0, 33, 0])
    case.set_old_from_oracle(oracle)
    fwd, dx, dw = run_fwd_bwd(spo, case, one_call=one_call)
    check_forward(case, oracle, fwd)
    rb = oracle.pg_loss_bwd(*case.oracle_inputs(), *case.eps)
    assert rel_l2(f64(dx), rb["d_hidden"]) < GRAD_TOL and rel_l2(f64(dw), rb["d_W"]) < GRAD_TOL
    say("fused: no tokens at all")
    case = Case(MID, [0, 0])
    case.old = np.zeros(0, np.float32)
    desc = case.to_gpu(spo)
    dW = torch.full((MID.V, MID.H), 7.0, device="cuda")
    if one_call:
        loss, logp, lse, stats, _, _ = spo.spo_pg_loss_fwd_bwd(desc, 1.0, d_W=dW, want_d_hidden=False)
    else:
        loss, logp, lse, stats = spo.spo_pg_loss_fwd(desc)
        spo.spo_pg_loss_bwd(desc, logp, lse, 1.0, d_W=dW, want_d_hidden=False)
    torch.cuda.synchronize()
    assert loss.item() == 0.0 and stats[0].item() == 0.0 and not dW.any()


@pytest.mark.parametrize("dtype,V", [("bf16", 3000), ("bf16", 1001), ("fp32", 3000), ("fp32", 1001)])
def test_logits_in_matches_oracle(spo, oracle, dtype, V):
    say(f"logits-in {dtype} T=713 V={V}")
    cfg = wl.scaled(MID, V=V, dtype=dtype)
    case = Case(cfg, MID_LENGTHS, mask_frac=0.25)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    # the logits a model would hand over, rounded to the storage type: they are the input
    logits = (case.hidden.float() @ case.W.float().t() * 4.0).to(tdt)
    lg64 = f64(logits)
    h, w, tg, _, mk, ad, cu = case.oracle_inputs()
    logp = oracle.pg_loss_fwd(None, None, tg, np.zeros(case.T), mk, ad, cu, *case.eps, logits=lg64)["logp"]
    old = (logp + case.noise).astype(np.float32)
    ratio = np.exp(logp - old)
    near = (np.abs(ratio - 0.8) < 2e-3) | (np.abs(ratio - 1.28) < 3e-3)
    old[near] += np.float32(0.01)
    case.old = old
    ref = oracle.pg_loss_fwd(None, None, tg, old.astype(np.float64), mk, ad, cu, *case.eps, logits=lg64)
    rb = oracle.pg_loss_bwd(None, None, tg, old.astype(np.float64), mk, ad, cu, *case.eps, logits=lg64)
    desc = case.to_gpu(spo, logits=logits.cuda())
    fwd = spo.spo_pg_loss_fwd(desc)
    dl = spo.spo_pg_loss_bwd(desc, fwd[1], fwd[2], 1.0)
    torch.cuda.synchronize()
    check_forward(case, oracle, fwd, ref=ref, atol_logp=2e-5 if dtype == "fp32" else 2e-4,
                  rtol_loss=2e-3)
    assert rel_l2(f64(dl), rb["d_logits"]) < (1e-5 if dtype == "fp32" else GRAD_TOL)
    assert not dl[torch.as_tensor(case.mask == 0)].any()


def test_target_id_out_of_range_gives_nan_not_garbage(spo, oracle):
    # sampled-token ids are not validated on the host; an id outside [0, V) must neither read out of
    # bounds nor leave a stale number behind: the token's log-prob is NaN, all other tokens are untouched
    say("fused and logits-in: one target id outside the vocabulary")
    case = Case(MID, MID_LENGTHS)
    case.set_old_from_oracle(oracle)
    ref = oracle.pg_loss_fwd(*case.oracle_inputs(), *case.eps)
    bad = np.array([5, 300, 712])
    good = np.setdiff1d(np.arange(case.T), bad)
    case.target = case.target.copy()
    case.target[bad] = [MID.V, -1, 2 ** 31 - 1]
    for logits in (None, (case.hidden.float() @ case.W.float().t()).to(torch.bfloat16).cuda()):
        loss, logp, lse, _ = spo.spo_pg_loss_fwd(case.to_gpu(spo, logits=logits))
        torch.cuda.synchronize()
        lp = f64(logp)
        assert np.isnan(lp[bad]).all() and np.isnan(loss.item())
        if logits is None:
            np.testing.assert_allclose(lp[good], ref["logp"][good], atol=2e-4, rtol=0)
            np.testing.assert_allclose(f64(lse), ref["lse"], atol=2e-4, rtol=0)
        else:
            assert np.isfinite(lp[good]).all() and np.isfinite(f64(lse)).all()
