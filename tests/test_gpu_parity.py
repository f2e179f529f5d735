"""GPU parity: the HIP draft/verify path against the CPU oracle (needs an MI355X)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2505_08600_amd import api
from paper_2505_08600_amd import datagen as dg

import sdharness as H

pytestmark = pytest.mark.gpu

TINY_T, TINY_D = dg.SHAPES["tiny_target"], dg.SHAPES["tiny_draft"]
# bf16 test models scale the LM head so that logits have the spread of the 7B-shape target
# (std 0.02*sqrt(4096) = 1.28 = 0.02*4*sqrt(256)): probability errors then relate to bf16
# rounding as they do at full size.  (The x20 scaling belongs to the fp32 config 1 only.)
BF16_LM_SCALE = 4.0


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def tiny_pair():
    p = H.Pair(TINY_T, TINY_D, seed=11, lm_scale=20.0)
    yield p
    p.close()


@pytest.fixture(scope="module")
def tiny_pair_bf16():
    p = H.Pair(dg.SHAPES["tiny_target_bf16"], dg.SHAPES["tiny_draft_bf16"], seed=12, lm_scale=BF16_LM_SCALE)
    yield p
    p.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_config1_tiny_fp32_teacher_forced(tiny_pair, T):
    """BASELINE config 1: tiny fp32 pair, gamma=4, prompt 32, 64 tokens."""
    _say(f"config1 fp32 T={T}")
    prompt = dg.make_prompt(11, 0, 32, TINY_T.vocab)
    st = H.teacher_forced_parity(tiny_pair, prompt, gamma=4, T=T, n_tokens=64, seed=11)
    _say(f"  steps={st.steps} flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} q_abs={st.max_q_abs:.2e}")
    assert st.flagged <= 1 and st.max_logit_rel < 1e-4


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_config1_tiny_fp32_free_running(tiny_pair, T):
    """Production loop (commit inside verify, no host reads between calls): emitted
    tokens equal the oracle's up to the oracle's first low-margin decision."""
    _say(f"config1 free-running T={T}")
    prompt = dg.make_prompt(11, 1, 32, TINY_T.vocab)
    toks, steps, _ = H.oracle_trajectory(tiny_pair, prompt, 4, T, 64, seed=23, keep_logits=False)
    got, n_steps, n_acc = H.free_running(tiny_pair, prompt, 4, T, 64, seed=23)
    # fp32 inverse-CDF sums differ from the oracle's fp64 ones by ~1e-7 of the mass; a step whose
    # margin is above 2e-6 cannot legitimately differ
    thr = 2e-6 if T > 0 else H.GREEDY_GAP_THR[dg.FP32]
    safe = 0
    for s in steps:
        if min(s.draft_margins.min(), s.verify_margins.min()) < thr:
            break
        safe += s.n_acc + 1
    safe = min(safe, 64)
    assert safe >= 32, "trajectory hits a low-margin decision too early to be a useful check"
    assert got[:safe] == toks[:safe]
    assert n_acc[:3] == [s.n_acc for s in steps[:3]]


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_perturbed_draft_exercises_partial_acceptance(T):
    """A draft that is a noisy copy of the target accepts 0 < n_acc < gamma often."""
    _say(f"perturbed draft T={T}")
    wt = dg.make_weights(TINY_T, 31, 20.0)
    wd = dg.perturbed_copy(wt, TINY_T, seed=32, rel=0.1)
    pair = H.Pair(TINY_T, TINY_T, 31, target_weights=wt, draft_weights=wd)
    prompt = dg.make_prompt(31, 0, 17, TINY_T.vocab)
    st = H.teacher_forced_parity(pair, prompt, gamma=5, T=T, n_tokens=48, seed=31)
    _say(f"  n_acc={st.n_acc} flagged={st.flagged}")
    assert len(set(st.n_acc)) >= 3 and st.flagged <= 1
    pair.close()


def test_target_as_its_own_draft_accepts_everything():
    """Exercises the two-row catch-up of the draft after fully accepted steps."""
    _say("draft == target")
    wt = dg.make_weights(TINY_T, 41, 20.0)
    pair = H.Pair(TINY_T, TINY_T, 41, target_weights=wt, draft_weights=wt)
    prompt = dg.make_prompt(41, 0, 9, TINY_T.vocab)
    for T in (0.0, 0.8):
        st = H.teacher_forced_parity(pair, prompt, gamma=3, T=T, n_tokens=24, seed=41)
        assert all(a == 3 for a in st.n_acc)
    got, _, n_acc = H.free_running(pair, prompt, 3, 0.0, 24, seed=41)
    ar, _ = oracle.ar_generate(pair.ot.new_seq(64), prompt, 0.0, 24, H.uf(41, dg.VERIFY_STREAM))
    assert got == ar and all(a == 3 for a in n_acc)
    pair.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_tiny_bf16_teacher_forced(tiny_pair_bf16, T):
    _say(f"tiny bf16 T={T}")
    prompt = dg.make_prompt(12, 0, 32, TINY_T.vocab)
    st = H.teacher_forced_parity(tiny_pair_bf16, prompt, gamma=4, T=T, n_tokens=64, seed=12)
    _say(f"  steps={st.steps} flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} q_abs={st.max_q_abs:.2e}")
    assert st.flagged <= H.flag_cap(st.steps) and st.max_logit_rel < 2e-2


@pytest.mark.parametrize("T,plen,gamma", [(0.0, 70, 5), (1.0, 70, 5), (1.0, 300, 8), (0.0, 33, 15)])
def test_small_bf16_mfma_kernels_teacher_forced(T, plen, gamma):
    """bf16 pair whose shapes take the MFMA GEMM and attention kernels (head_dim 128
    target, 64 draft); prompts span several KV tiles, splits and a ragged tail."""
    _say(f"small bf16 (MFMA path) T={T} prompt={plen} gamma={gamma}")
    st_, sd_ = dg.SHAPES["small_target_bf16"], dg.SHAPES["small_draft_bf16"]
    pair = H.Pair(st_, sd_, seed=61, lm_scale=BF16_LM_SCALE, max_rows=32, max_pos=512)
    prompt = dg.make_prompt(61, plen, plen, st_.vocab)
    st = H.teacher_forced_parity(pair, prompt, gamma=gamma, T=T, n_tokens=40, seed=61 + plen)
    _say(f"  steps={st.steps} flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} q_abs={st.max_q_abs:.2e}")
    assert st.flagged <= H.flag_cap(st.steps) and st.max_logit_rel < 2e-2
    pair.close()


@pytest.mark.parametrize("dtype,T", [(dg.FP32, 1.0), (dg.BF16, 1.0), (dg.BF16, 0.0)])
def test_largest_vocabulary_teacher_forced(dtype, T):
    """Vocabulary 262144, the largest sd_load_model accepts: the samplers' table of 64 segments of 4096 entries is
    full, the draft sampler and the verify tail take their general (strided) kernels, a logits row is 1 MB.  One
    layer of width 64, a few steps along the oracle's trajectory."""
    _say(f"largest vocabulary, dtype={dtype} T={T}")
    V = 262144
    st_ = dg.ModelShape("vmax_t", 1, 64, 1, 64, 128, V, dtype)
    sd_ = dg.ModelShape("vmax_d", 1, 64, 1, 64, 64, V, dtype)
    pair = H.Pair(st_, sd_, seed=71, lm_scale=BF16_LM_SCALE if dtype == dg.BF16 else 20.0, max_rows=32, max_pos=128)
    prompt = dg.make_prompt(71, 0, 19, V)
    st = H.teacher_forced_parity(pair, prompt, gamma=3, T=T, n_tokens=10, seed=71)
    _say(f"  steps={st.steps} flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} q_abs={st.max_q_abs:.2e}")
    # (a token of this vocabulary holds about 4e-6 of the mass, a few float32 steps of the running sum: a draw may
    # land on the neighbouring token, which the decision rule allows and counts)
    assert st.flagged <= 2 and st.max_logit_rel < (2e-2 if dtype == dg.BF16 else 1e-4)
    pair.close()


def test_small_bf16_every_prompt_length_across_the_first_tiles():
    """Every prompt length from 1 (nothing to prefill: the first pass starts on an empty cache) to 100 tokens: the
    cache length at the first verify pass takes every position
    inside the first three 32-token K / V tiles (tile starts and ends included), with gamma + 1 = 5 new rows that
    straddle a tile boundary in every fourth case; two steps each, teacher-forced, T = 1."""
    _say("small bf16: prompt lengths 1..100")
    st_, sd_ = dg.SHAPES["small_target_bf16"], dg.SHAPES["small_draft_bf16"]
    pair = H.Pair(st_, sd_, seed=63, lm_scale=BF16_LM_SCALE, max_rows=32, max_pos=160)
    flagged = steps = 0
    worst = 0.0
    for plen in range(1, 101):
        prompt = dg.make_prompt(63, plen, plen, st_.vocab)
        st = H.teacher_forced_parity(pair, prompt, gamma=4, T=1.0, n_tokens=4, seed=63 + plen)
        flagged += st.flagged
        steps += st.steps
        worst = max(worst, st.max_logit_rel)
    _say(f"  steps={steps} flagged={flagged} logit_rel={worst:.2e}")
    assert flagged <= H.flag_cap(steps) and worst < 2e-2
    pair.close()


def test_small_bf16_mfma_matches_reference_kernels():
    """The MFMA kernels and the simple reference kernels of the library agree to bf16
    rounding on the same inputs (both are also compared with the oracle elsewhere)."""
    _say("small bf16: MFMA vs reference kernels")
    st_, sd_ = dg.SHAPES["small_target_bf16"], dg.SHAPES["small_draft_bf16"]
    pair = H.Pair(st_, sd_, seed=62, lm_scale=BF16_LM_SCALE, max_rows=32, max_pos=512)
    prompt = dg.make_prompt(62, 0, 150, st_.vocab)
    outs = []
    for force in (0, 1):
        api.set_option("force_generic", force)
        try:
            ctx = api.Context([256])
            ctx.attach(pair.gt)
            H.gpu_prefill(ctx, [pair.gt], [list(prompt)])
            na = torch.zeros(1, dtype=torch.int32, device="cuda")
            nx = torch.zeros(1, dtype=torch.int32, device="cuda")
            cand = H.dev(np.array([[5, 6, 7, 8, 9]], np.int32))
            api.sd_verify(pair.gt, ctx, None, 1, 5, 0.0, cand, None, None, na, nx, commit=False)
            outs.append(pair.gt.last_logits().cpu().numpy())
            ctx.close()
        finally:
            api.set_option("force_generic", 0)
    rel = np.abs(outs[0] - outs[1]).max() / np.abs(outs[1]).max()
    _say(f"  rel diff {rel:.2e}")
    assert rel < 5e-3
    pair.close()


@pytest.mark.parametrize("B", [2, 3, 5, 8, 11, 16, 17, 30])
def test_small_bf16_every_gemm_row_class_matches_reference_kernels(B):
    """Batched verify at gamma = 5 with B ragged sequences puts M = 6B rows through every GEMM: the packed
    (M <= 8), 16- and 32-row few-row kernels, the 48-row blocks (M <= 64) and the 96-row blocks, with ragged
    last blocks, plus batched prefill chunks.  The MFMA path must agree with the library's reference
    kernels (which the oracle tests pin) far inside the bf16 tolerance: both feed hi + lo activations."""
    _say(f"small bf16: batch {B} (M = {6 * B}) MFMA vs reference kernels")
    st_ = dg.SHAPES["small_target_bf16"]
    w = dg.make_weights(st_, 63, BF16_LM_SCALE)
    gt = api.Model(st_, w, max_rows=max(32, 6 * B), max_pos=256)
    lens = dg.make_prompt_lengths(63 + B, B, 5, 90)
    prompts = [[int(t) for t in dg.make_prompt(63, b, int(lens[b]), st_.vocab)] for b in range(B)]
    cand = H.dev(dg.make_prompt(64, B, 5 * B, st_.vocab).reshape(B, 5).astype(np.int32))
    outs = []
    for force in (0, 1):
        api.set_option("force_generic", force)
        try:
            ctx = api.Context([int(l) + 16 for l in lens])
            ctx.attach(gt)
            H.gpu_prefill(ctx, [gt], prompts)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            api.sd_verify(gt, ctx, None, B, 5, 0.0, cand, None, None, na, nx, commit=False)
            ctx.sync()
            outs.append((gt.last_logits().cpu().numpy(), na.cpu().numpy().copy(), nx.cpu().numpy().copy()))
            if force == 0:  # attention blocks start longest sequence first (ties: lower slot first)
                order = gt.debug_read("seq_order", B)[:, 0].astype(int)
                ln = gt.debug_read("seq_len", B)[:, 0].astype(int)
                assert (ln == lens - 1 + 6).all()
                assert order.tolist() == sorted(range(B), key=lambda b: (-ln[b], b))
            ctx.close()
        finally:
            api.set_option("force_generic", 0)
    rel = np.abs(outs[0][0] - outs[1][0]).max() / np.abs(outs[1][0]).max()
    _say(f"  rel diff {rel:.2e}")
    assert outs[0][0].shape == (6 * B, st_.vocab) and np.isfinite(outs[0][0]).all()
    assert rel < 2e-3
    gt.close()


@pytest.mark.parametrize("cols,B", [(192, 16), (192, 20), (192, 30), (256, 20), (256, 30), (128, 16), (128, 20), (128, 30)])
def test_small_bf16_row_blocked_gemm_block_widths_match_reference_kernels(cols, B):
    """The 96- and 64-row GEMM blocks (64 rows at batch 20: M = 120 pads less that way) are 256, 192 or (plain
    projections with a short K only) 128 weight rows wide; the library picks by how well the blocks fill the chip,
    so each width is forced here.  d_ffn = 896 gives the 192-row SwiGLU blocks (96 output
    columns, gate/up pairs straddling waves) a partial last block: 896 = 9 * 96 + 32."""
    import dataclasses
    _say(f"small bf16: 96-row GEMM blocks forced to {cols} weight rows, batch {B}, d_ffn 896")
    st_ = dataclasses.replace(dg.SHAPES["small_target_bf16"], d_ffn=896, name="small_target_bf16_f896")
    w = dg.make_weights(st_, 67, BF16_LM_SCALE)
    gt = api.Model(st_, w, max_rows=6 * B, max_pos=256)
    lens = dg.make_prompt_lengths(71 + B, B, 5, 90)
    prompts = [[int(t) for t in dg.make_prompt(67, b, int(lens[b]), st_.vocab)] for b in range(B)]
    cand = H.dev(dg.make_prompt(68, B, 5 * B, st_.vocab).reshape(B, 5).astype(np.int32))
    outs = []
    for force in (0, 1):
        api.set_option("force_generic", force)
        api.set_option("gemm_tile_cols", 0 if force else cols)
        try:
            ctx = api.Context([int(l) + 16 for l in lens])
            ctx.attach(gt)
            H.gpu_prefill(ctx, [gt], prompts)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            api.sd_verify(gt, ctx, None, B, 5, 0.0, cand, None, None, na, nx, commit=False)
            ctx.sync()
            outs.append((gt.last_logits().cpu().numpy(), gt.debug_read("act", 6 * B)))
            ctx.close()
        finally:
            api.set_option("force_generic", 0)
            api.set_option("gemm_tile_cols", 0)
    rel = np.abs(outs[0][0] - outs[1][0]).max() / np.abs(outs[1][0]).max()
    rel_act = np.abs(outs[0][1] - outs[1][1]).max() / np.abs(outs[1][1]).max()
    _say(f"  rel diff logits {rel:.2e}, SwiGLU output of the last layer {rel_act:.2e}")
    assert np.isfinite(outs[0][0]).all() and rel < 2e-3 and rel_act < 2e-3
    gt.close()


@pytest.mark.parametrize("waves", [4, 8])
def test_small_bf16_both_fused_attention_block_shapes_match_reference_kernels(waves):
    """The fused attention kernel runs as 8-wave blocks (few sequences) or 4-wave blocks (many); the
    library picks by batch size, so each shape is forced here on the same ragged batch and compared with
    the reference kernels."""
    _say(f"small bf16: fused attention forced to {waves}-wave blocks vs reference kernels")
    st_ = dg.SHAPES["small_target_bf16"]
    w = dg.make_weights(st_, 65, BF16_LM_SCALE)
    B = 6
    gt = api.Model(st_, w, max_rows=6 * B, max_pos=256)
    lens = dg.make_prompt_lengths(70, B, 5, 200)
    prompts = [[int(t) for t in dg.make_prompt(65, b, int(lens[b]), st_.vocab)] for b in range(B)]
    cand = H.dev(dg.make_prompt(66, B, 5 * B, st_.vocab).reshape(B, 5).astype(np.int32))
    outs = []
    for force in (0, 1):
        api.set_option("force_generic", force)
        api.set_option("attn_waves", 0 if force else waves)
        try:
            ctx = api.Context([int(l) + 16 for l in lens])
            ctx.attach(gt)
            H.gpu_prefill(ctx, [gt], prompts)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            api.sd_verify(gt, ctx, None, B, 5, 0.0, cand, None, None, na, nx, commit=False)
            ctx.sync()
            outs.append(gt.last_logits().cpu().numpy())
            ctx.close()
        finally:
            api.set_option("force_generic", 0)
            api.set_option("attn_waves", 0)
    rel = np.abs(outs[0] - outs[1]).max() / np.abs(outs[1]).max()
    _say(f"  rel diff {rel:.2e}")
    assert np.isfinite(outs[0]).all() and rel < 2e-3
    gt.close()


@pytest.mark.parametrize("T,plen,gamma", [(0.0, 70, 5), (1.0, 70, 5), (1.0, 300, 4), (0.0, 33, 7)])
def test_small_bf16_norm_split_between_its_neighbour_gemms_matches_oracle(T, plen, gamma):
    """With few rows the add + RMSNorm launches of a layer can be split between the projection before them (which
    adds the residual, applies the gains and leaves per-block sums of squares) and the GEMM after them (which
    scales its sums by 1 / rms): the operand is then rounded to its two bf16 terms before the division by rms
    instead of after it.  This is the library's default where the shapes allow; option norm_fold = 2 switches it
    off, and the same oracle comparison must hold both ways, with the same limits (target and draft both take
    the path, draft rows included: 1-2 rows, LM head through a row map)."""
    _say(f"small bf16, split norm, T={T} prompt={plen} gamma={gamma}")
    st_, sd_ = dg.SHAPES["small_target_bf16"], dg.SHAPES["small_draft_bf16"]
    pair = H.Pair(st_, sd_, seed=61, lm_scale=BF16_LM_SCALE, max_rows=32, max_pos=512)
    prompt = dg.make_prompt(61, plen, plen, st_.vocab)
    for opt in (1, 2):
        api.set_option("norm_fold", opt)
        try:
            st = H.teacher_forced_parity(pair, prompt, gamma=gamma, T=T, n_tokens=40, seed=61 + plen)
        finally:
            api.set_option("norm_fold", 0)
        _say(f"  norm_fold={opt}: steps={st.steps} flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} q_abs={st.max_q_abs:.2e}")
        assert st.flagged <= H.flag_cap(st.steps) and st.max_logit_rel < 2e-2
    pair.close()


@pytest.mark.parametrize("shape_name,B", [("small_target_bf16", 1), ("small_target_bf16", 5), ("small_draft_bf16", 3),
                                          ("draft_a_1layer", 1)])
def test_norm_split_between_its_neighbour_gemms_matches_the_norm_launches(shape_name, B):
    """The same forward with the split norm on (the default) and off (option norm_fold = 2): the logits differ
    by the rounding of the operand at another point only - a few 1e-5 of their range at these widths, four orders
    of magnitude inside the tolerance; 1 to 30 rows (packed, 16- and 32-row kernels)."""
    import dataclasses
    _say(f"{shape_name}: split norm vs norm launches, batch {B}")
    st_ = (dataclasses.replace(dg.SHAPES["draft_a"], n_layers=1, vocab=2048, name="draft_a_1layer")
           if shape_name == "draft_a_1layer" else dg.SHAPES[shape_name])
    w = dg.make_weights(st_, 81, BF16_LM_SCALE)
    gt = api.Model(st_, w, max_rows=max(16, 6 * B), max_pos=256)
    lens = dg.make_prompt_lengths(81 + B, B, 5, 150)
    prompts = [[int(t) for t in dg.make_prompt(81, b, int(lens[b]), st_.vocab)] for b in range(B)]
    cand = H.dev(dg.make_prompt(82, B, 5 * B, st_.vocab).reshape(B, 5).astype(np.int32))
    outs = []
    for opt in (2, 1):
        api.set_option("norm_fold", opt)
        try:
            ctx = api.Context([int(l) + 16 for l in lens])
            ctx.attach(gt)
            H.gpu_prefill(ctx, [gt], prompts)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            api.sd_verify(gt, ctx, None, B, 5, 0.0, cand, None, None, na, nx, commit=False)
            ctx.sync()
            outs.append(gt.last_logits().cpu().numpy())
            ctx.close()
        finally:
            api.set_option("norm_fold", 0)
    rel = np.abs(outs[0] - outs[1]).max() / np.abs(outs[0]).max()
    _say(f"  rel diff {rel:.2e}")
    assert np.isfinite(outs[1]).all() and rel < 2e-4
    assert not np.array_equal(outs[0], outs[1]), "the option did not change the path"
    gt.close()


@pytest.mark.parametrize("shape_name,B", [("small_target_bf16", 1), ("small_target_bf16", 5), ("small_draft_bf16", 3),
                                          ("draft_a_1layer", 1), ("draft_a_1layer", 2)])
def test_attention_blocks_applying_the_output_projection_match_the_separate_launch(shape_name, B):
    """For small models in few blocks the fused attention kernel multiplies its head's output rows with that
    head's columns of the output projection and leaves one partial slab per head for the add + norm kernel
    (head widths 128 and 64; 2, 2 and 12 heads).  Option force_generic = 8 takes the projection out again as a
    GEMM launch of its own; both orders of the same fp32 sums must agree far inside the bf16 tolerance."""
    import dataclasses
    _say(f"{shape_name}: output projection inside the attention blocks vs its own launch, batch {B}")
    st_ = (dataclasses.replace(dg.SHAPES["draft_a"], n_layers=1, vocab=2048, name="draft_a_1layer")
           if shape_name == "draft_a_1layer" else dg.SHAPES[shape_name])
    w = dg.make_weights(st_, 81, BF16_LM_SCALE)
    gt = api.Model(st_, w, max_rows=max(16, 6 * B), max_pos=256)
    lens = dg.make_prompt_lengths(81 + B, B, 5, 150)
    prompts = [[int(t) for t in dg.make_prompt(81, b, int(lens[b]), st_.vocab)] for b in range(B)]
    cand = H.dev(dg.make_prompt(82, B, 5 * B, st_.vocab).reshape(B, 5).astype(np.int32))
    outs = []
    for force in (0, 8):
        api.set_option("force_generic", force)
        api.set_option("norm_fold", 2)  # (with the split norm the projection is a launch of its own anyway)
        try:
            ctx = api.Context([int(l) + 16 for l in lens])
            ctx.attach(gt)
            H.gpu_prefill(ctx, [gt], prompts)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            api.sd_verify(gt, ctx, None, B, 5, 0.0, cand, None, None, na, nx, commit=False)
            ctx.sync()
            outs.append(gt.last_logits().cpu().numpy())
            ctx.close()
        finally:
            api.set_option("force_generic", 0)
            api.set_option("norm_fold", 0)
    rel = np.abs(outs[0] - outs[1]).max() / np.abs(outs[1]).max()
    _say(f"  rel diff {rel:.2e}")
    assert outs[0].shape == (6 * B, st_.vocab) and np.isfinite(outs[0]).all() and rel < 2e-4
    assert not np.array_equal(outs[0], outs[1]), "the option did not change the path"
    gt.close()


@pytest.mark.parametrize("force", [0, 4])
def test_draft_candidates_for_uniforms_on_the_boundaries_of_q(force):
    """Both draft samplers (one block per 2048-column slice working from the LM head's partials; one block per row,
    option force_generic = 4) place u * Z with sums added in parallel - per thread of four consecutive columns, per
    wave of 256, per slice - and where two partial sums disagree by rounding the candidate must still be one of the
    two tokens whose intervals meet there (Section 3.1: candidates are draws from q).  30 sequences with the same
    prompt give 30 draws from one q per call (few enough rows for the LM head to leave its partials); their uniforms sit on, or one float32 step beside, the thread, wave
    and slice ends of the CDF of the q row the sampler itself wrote.  Each candidate must lie within 1e-5 of u in
    that CDF and have positive q."""
    import dataclasses
    _say(f"small bf16 draft: candidates for uniforms on the ends of partial sums, force_generic={force}")
    sd_ = dataclasses.replace(dg.SHAPES["small_draft_bf16"], vocab=6176, name="small_draft_v6176")
    w = dg.make_weights(sd_, 84, BF16_LM_SCALE)
    B, V, T = 30, sd_.vocab, 0.9
    gd = api.Model(sd_, w, max_rows=2 * B, max_pos=64)
    prompt = [int(t) for t in dg.make_prompt(84, 0, 23, V)]
    rng = np.random.default_rng(84)
    api.set_option("force_generic", force)
    try:
        ctx = api.Context([40] * B)
        ctx.attach(gd)
        H.gpu_prefill(ctx, [gd], [prompt] * B)
        cand = torch.full((B, 1), -1, dtype=torch.int32, device="cuda")
        q = torch.zeros((B, 1, V), dtype=torch.float32, device="cuda")

        def draw(u):
            api.sd_draft(gd, ctx, None, B, 1, T, H.dev(u.reshape(B, 1).astype(np.float32)), cand, q)
            ctx.sync()
            for b in range(B):
                ctx.truncate(gd, b, len(prompt) - 1)
            return cand.cpu().numpy()[:, 0].copy(), q.cpu().numpy()[:, 0].copy()

        _, q0 = draw(np.full(B, 0.5))
        assert all(np.array_equal(q0[b], q0[0]) for b in range(B)), "equal prompts must give equal q rows"
        qd = q0[0].astype(np.float64)
        cdf = np.cumsum(qd) / qd.sum()
        other = trials = 0
        for ends in (np.arange(3, V - 4, 4), np.arange(255, V - 4, 256), np.arange(2047, V - 4, 2048)) * 8:
            ks = rng.choice(ends, B // 3)
            us = np.concatenate([[np.float32(cdf[k]), np.nextafter(np.float32(cdf[k]), np.float32(0)),
                                  np.nextafter(np.float32(cdf[k]), np.float32(1))] for k in ks]).astype(np.float32)
            us = np.clip(us, np.float32(2.0 ** -24), np.float32(1.0 - 2.0 ** -24))
            c, q1 = draw(us)
            assert np.array_equal(q1, q0)
            for b in range(B):
                trials += 1
                ref = oracle.sample_cdf(qd, float(us[b]))[0]
                if int(c[b]) != ref:
                    other += 1
                    assert 0 <= c[b] < V and qd[c[b]] > 0, (b, int(c[b]), ref)
                    d = oracle.cdf_distance(qd, float(us[b]), int(c[b]))
                    assert d < 1e-5, (b, float(us[b]), int(c[b]), ref, d)
        _say(f"  {trials} uniforms, {other} resolved to the neighbouring token")
        ctx.close()
    finally:
        api.set_option("force_generic", 0)
    gd.close()


@pytest.mark.parametrize("dist", [1, 32, 3088])
@pytest.mark.parametrize("force", [0, 4])
def test_greedy_draft_with_every_logit_twice_takes_the_lower_token(force, dist):
    """T = 0 with an LM head in which token t + dist has the same row as token t (for every t whose index / dist is
    even): every logit, the largest included, occurs twice - next to each other, one 32-column partial apart, or half
    the vocabulary apart - and the greedy candidate must be the lower of the two, as the oracle's arg max is.  Both
    draft samplers (from the LM head's partials; one block per row with option force_generic = 4)."""
    import dataclasses
    _say(f"small bf16 draft: greedy with duplicated logits at distance {dist}, force_generic={force}")
    sd_ = dataclasses.replace(dg.SHAPES["small_draft_bf16"], vocab=6176, name="small_draft_v6176")
    w = dict(dg.make_weights(sd_, 85, BF16_LM_SCALE))
    V, B, gamma = sd_.vocab, 4, 6
    lm = np.array(w["lm_head"], copy=True)
    lower = (np.arange(V) // dist) % 2 == 0
    lower &= np.arange(V) + dist < V
    idx = np.nonzero(lower)[0]
    lm[idx + dist] = lm[idx]
    w["lm_head"] = lm
    gd = api.Model(sd_, w, max_rows=16, max_pos=128)
    od = oracle.OracleModel(sd_, w)
    prompts = [[int(t) for t in dg.make_prompt(85, b, 11 + 9 * b, V)] for b in range(B)]
    api.set_option("force_generic", force)
    try:
        ctx = api.Context([64] * B)
        ctx.attach(gd)
        H.gpu_prefill(ctx, [gd], prompts)
        cand = torch.full((B, gamma), -1, dtype=torch.int32, device="cuda")
        api.sd_draft(gd, ctx, None, B, gamma, 0.0, None, cand, None)
        ctx.sync()
        c = cand.cpu().numpy()
        ctx.close()
    finally:
        api.set_option("force_generic", 0)
    assert ((0 <= c) & (c < V)).all()
    upper = np.zeros(V, bool)
    upper[idx + dist] = True
    assert not upper[c].any(), ("a duplicate's upper copy was chosen", c)
    for b in range(B):   # and the candidates are the oracle's
        seq = od.new_seq(64)
        oracle.prefill(seq, prompts[b])
        ref, _, _ = seq.draft(prompts[b], gamma, 0.0, np.zeros(gamma, np.float32))
        assert list(c[b]) == [int(t) for t in ref], (b, c[b], ref)
    gd.close()


@pytest.mark.parametrize("T", [0.0, 0.9])
def test_draft_sampler_from_the_lm_heads_partials_matches_the_whole_row_sampler(T):
    """The LM head of a bf16 model leaves (max, sum of exponentials, arg-max) per 32 columns; the draft sampler
    then runs one block per 2048-column slice, none waiting for another, and the block that draws the token also
    gathers and norms the next forward's row.  Option force_generic = 4 brings back the sampler in which one
    block reads the whole row, and the embedding launch.  Vocabulary 6176 = 3 slices + 32 columns; three
    sequences, one of them with fewer candidates of its own; two draft calls in a row."""
    import dataclasses
    _say(f"small bf16 draft: sampler from LM-head partials vs whole-row sampler, T={T}")
    sd_ = dataclasses.replace(dg.SHAPES["small_draft_bf16"], vocab=6176, name="small_draft_v6176")
    w = dg.make_weights(sd_, 83, BF16_LM_SCALE)
    gd = api.Model(sd_, w, max_rows=16, max_pos=256)
    B, gamma, V = 3, 4, sd_.vocab
    prompts = [[int(t) for t in dg.make_prompt(83, b, 20 + 7 * b, V)] for b in range(B)]
    u = H.dev(np.stack([np.stack([dg.make_uniforms(83, dg.DRAFT_STREAM, b, k, gamma) for b in range(B)]) for k in range(2)]))
    outs = []
    for force in (0, 4):
        api.set_option("force_generic", force)
        try:
            ctx = api.Context([64] * B)
            ctx.attach(gd)
            H.gpu_prefill(ctx, [gd], prompts)
            ctx.policy_set([4, 2, 4])
            res = []
            for k in range(2):
                cand = torch.full((B, gamma), -1, dtype=torch.int32, device="cuda")
                q = torch.zeros((B, gamma, V), dtype=torch.float32, device="cuda")
                api.sd_draft(gd, ctx, None, B, gamma, T, u[k] if T > 0 else None, cand, q if T > 0 else None)
                ctx.sync()
                res.append((cand.cpu().numpy().copy(), q.cpu().numpy().copy(), gd.last_logits().cpu().numpy().copy()))
                for b in range(B):  # roll the draft cache back: the second call drafts from the same state
                    ctx.truncate(gd, b, len(prompts[b]) - 1)
            outs.append(res)
            ctx.close()
        finally:
            api.set_option("force_generic", 0)
    for k in range(2):
        (c0, q0, l0), (c1, q1, l1) = outs[0][k], outs[1][k]
        counts = [4, 2, 4]
        for b in range(B):
            assert (c0[b, :counts[b]] == c1[b, :counts[b]]).all(), (k, b, c0[b], c1[b])
            assert ((0 <= c0[b, :counts[b]]) & (c0[b, :counts[b]] < V)).all()
        assert np.array_equal(l0, l1), "the logits of the last forward must not depend on the sampler"
        if T > 0:
            for b in range(B):
                dq = np.abs(q0[b, :counts[b]] - q1[b, :counts[b]]).max()
                assert dq < 1e-6, (k, b, dq)
                assert np.abs(q0[b, :counts[b]].sum(-1) - 1.0).max() < 1e-4
    gd.close()


def test_draft_and_verify_are_graph_capturable_and_replays_match_eager():
    """sd_draft and sd_verify launch kernels only (no allocation, copy, memset or host synchronisation), so a
    caller may capture them into a HIP graph.  Every replay, with eager calls and synchronisations in
    between, must reproduce the eager results bit for bit."""
    _say("small bf16: graph capture of draft + verify")
    st_, sd_ = dg.SHAPES["small_target_bf16"], dg.SHAPES["small_draft_bf16"]
    pair = H.Pair(st_, sd_, seed=65, lm_scale=BF16_LM_SCALE, max_rows=32, max_pos=512)
    V, gamma, T = st_.vocab, 5, 1.0
    prompt = [int(t) for t in dg.make_prompt(65, 0, 100, V)]
    ctx = api.Context([256])
    ctx.attach(pair.gt)
    ctx.attach(pair.gd)
    H.gpu_prefill(ctx, [pair.gt, pair.gd], [prompt])
    ud = H.dev(dg.make_uniforms(65, dg.DRAFT_STREAM, 0, 0, gamma)[None])
    uv = H.dev(dg.make_uniforms(65, dg.VERIFY_STREAM, 0, 0, gamma + 1)[None])
    cand = torch.zeros((1, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((1, gamma, V), dtype=torch.float32, device="cuda")
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    nx = torch.zeros(1, dtype=torch.int32, device="cuda")

    def step():
        api.sd_draft(pair.gd, ctx, None, 1, gamma, T, ud, cand, q)
        api.sd_verify(pair.gt, ctx, None, 1, gamma, T, cand, q, uv, na, nx, commit=False)

    def rollback():
        torch.cuda.synchronize()
        ctx.truncate(pair.gt, 0, len(prompt) - 1)
        ctx.truncate(pair.gd, 0, len(prompt) - 1)

    def snapshot():
        torch.cuda.synchronize()
        return (cand.cpu().numpy().copy(), q.cpu().numpy().copy(), int(na.item()), int(nx.item()),
                pair.gt.last_logits().cpu().numpy().copy())

    step()
    ref = snapshot()
    rollback()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
        rollback()
        with torch.cuda.graph(graph, stream=side):
            step()
    rollback()
    for r in range(3):
        for t in (cand, q, na, nx):
            t.zero_()
        graph.replay()
        got = snapshot()
        rollback()
        for a, b in zip(ref, got):
            assert np.array_equal(np.asarray(a), np.asarray(b)), f"replay {r} differs from the eager step"
        step()  # the program's own eager work between replays
        got = snapshot()
        rollback()
        for a, b in zip(ref, got):
            assert np.array_equal(np.asarray(a), np.asarray(b))
    ctx.sync()
    ctx.close()
    pair.close()


def test_committing_graph_replayed_far_past_its_capture_time_lengths():
    """A graph of one committing greedy step (draft + verify with commit) of the fp32 pair - whose attention runs on
    the plain kernel, the one that sizes a score buffer on the host - is captured when the sequence holds 20 tokens
    and replayed until it holds more than three times that.  Launch sizes are those of capture time; results must
    not depend on them: the replays emit exactly the tokens of the same steps launched eagerly (which are the
    target's own greedy decoding, checked against the oracle), and no status flag is raised."""
    _say("fp32: committing graph replayed past the capture-time lengths")
    st_, sd_ = TINY_T, dg.SHAPES["tiny_draft"]
    wt = dg.make_weights(st_, 45, 20.0)
    pair = H.Pair(st_, st_, 45, target_weights=wt, draft_weights=dg.perturbed_copy(wt, st_, seed=46, rel=0.1))
    gamma, n_steps, V = 3, 24, st_.vocab
    prompt = [int(t) for t in dg.make_prompt(45, 0, 20, V)]
    cand = torch.zeros((1, gamma), dtype=torch.int32, device="cuda")
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    nx = torch.zeros(1, dtype=torch.int32, device="cuda")

    def new_ctx():
        c = api.Context([160])
        c.attach(pair.gt)
        c.attach(pair.gd)
        H.gpu_prefill(c, [pair.gt, pair.gd], [prompt])
        return c

    def step(c):
        api.sd_draft(pair.gd, c, None, 1, gamma, 0.0, None, cand, None)
        api.sd_verify(pair.gt, c, None, 1, gamma, 0.0, cand, None, None, na, nx, commit=True)

    ce = new_ctx()
    for _ in range(n_steps):
        step(ce)
    ce.sync()
    eager = list(ce.get_tokens(0))
    ce.close()
    cg = new_ctx()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(cg)
    for r in range(n_steps):
        graph.replay()
        if r % 5 == 4:   # eager work and synchronisations of the program between replays
            torch.cuda.synchronize()
            _ = cand.cpu()
    torch.cuda.synchronize()
    nt, kv = cg.sync(pair.gt)           # raises on any status flag
    got = list(cg.get_tokens(0))
    assert nt[0] == len(got) and kv[0] == nt[0] - 1
    assert len(got) >= 3 * len(prompt) or len(got) >= len(prompt) + n_steps
    assert got == eager, "graph replays and eager steps emitted different tokens"
    # and the tokens are the target's own greedy continuation (up to the oracle's first near-tie)
    ar, margins = oracle.ar_generate(pair.ot.new_seq(200), prompt, 0.0, len(got) - len(prompt), H.uf(45, dg.VERIFY_STREAM))
    safe = 0
    for mg in margins:
        if mg < H.GREEDY_GAP_THR[dg.FP32]:
            break
        safe += 1
    assert safe >= 20 and got[len(prompt):len(prompt) + safe] == ar[:safe]
    cg.close()
    pair.close()


@pytest.mark.parametrize("shape_name,tol,max_rows,lens", [
    ("tiny_target", 1e-4, 96, [9, 41, 150]), ("small_target_bf16", 2e-2, 96, [9, 41, 150]),
    ("small_target_bf16", 2e-2, 144, [9, 41, 150]), ("small_target_bf16", 2e-2, 192, [9, 41, 150]),
    ("small_target_bf16", 2e-2, 576, [1000, 333, 17]),   # 12 groups per sequence and forward
    ("small_target_bf16", 2e-2, 288, [1000, 333, 17]),   # 6 groups: the second block of four holds two
    ("small_draft_bf16", 2e-2, 192, [1000, 70, 129])])   # head width 64, several forwards
def test_prefill_in_row_groups_matches_oracle(shape_name, tol, max_rows, lens):
    """With a workspace of 96 rows sd_prefill feeds three ragged prompts in groups of 16 rows, two groups
    per sequence and forward (plan slots), through the separate cache-append and attention kernels; prompt
    lengths cover an empty second group, a partial one and several forwards.  The cache it leaves must
    give the oracle's logits in the verify pass that follows, and the oracle's decisions.  With 144 and 192
    rows there are three and four groups per sequence; the 1000-token prompts take several forwards of up to
    twelve groups."""
    _say(f"prefill in row groups, {shape_name}, workspace {max_rows} rows, prompts {lens}")
    st_ = dg.SHAPES[shape_name]
    w = dg.make_weights(st_, 81, BF16_LM_SCALE if st_.dtype == dg.BF16 else 1.0)
    om = oracle.OracleModel(st_, w)
    gm = api.Model(st_, w, max_rows=max_rows, max_pos=max(lens) + 64)
    gamma, V = 3, st_.vocab
    prompts = [[int(t) for t in dg.make_prompt(81, b, n, V)] for b, n in enumerate(lens)]
    ctx = api.Context([n + 16 for n in lens])
    ctx.attach(gm)
    H.gpu_prefill(ctx, [gm], prompts)
    nt, kv = ctx.sync(gm)
    assert list(nt) == lens and list(kv) == [n - 1 for n in lens]
    cand = dg.make_prompt(82, 0, 3 * gamma, V).reshape(3, gamma).astype(np.int32)
    na = torch.zeros(3, dtype=torch.int32, device="cuda")
    nx = torch.zeros(3, dtype=torch.int32, device="cuda")
    api.sd_verify(gm, ctx, None, 3, gamma, 0.0, H.dev(cand), None, None, na, nx, commit=False)
    lg = gm.last_logits().cpu().numpy().reshape(3, gamma + 1, V)
    for b in range(3):
        seq = om.new_seq(lens[b] + 16)
        oracle.prefill(seq, prompts[b])
        r_na, r_nx, mg, r_lg = seq.verify(prompts[b], gamma, 0.0, cand[b], None, np.zeros(gamma + 1, np.float32),
                                          want_logits=True)
        rel = np.abs(lg[b] - r_lg).max() / np.abs(r_lg).max()
        _say(f"  sequence {b} (prompt {lens[b]}): logits rel err {rel:.2e}")
        assert rel < tol
        if (int(na[b]), int(nx[b])) != (r_na, r_nx):   # greedy: only a top-1/top-2 gap below the flat threshold may flip
            i = min(r_na, int(na[b]))
            assert mg[i] < H.MARGIN_THR[st_.dtype] * np.abs(r_lg[i]).max(), (b, na[b], nx[b], r_na, r_nx, mg)
    ctx.close()
    gm.close()


@pytest.mark.parametrize("shape_name,max_rows,lens", [("small_target_bf16", 112, [700]), ("draft_a_1layer", 160, [333, 650]),
                                                      ("small_draft_bf16", 64, [200, 90])])
def test_prefill_attention_sharing_tiles_between_row_groups_matches_the_split_kernel(shape_name, max_rows, lens):
    """Prefill forwards send four 16-row groups of a prompt and head to one block, which stages every K / V
    tile in LDS once for its four waves (and splits the tile range over several blocks plus a combine pass when
    there are few blocks).  Option prefill_attn = 0 brings back one set of split-kernel blocks per group.  Both
    compute the same softmax in other partitions: the verify logits after the prefill agree to rounding level.
    Seven, five and two groups per sequence and forward: blocks whose last waves have no group, and whose
    groups end at different tiles."""
    import dataclasses
    _say(f"{shape_name}: prefill attention with shared tiles vs split kernel, workspace {max_rows}, prompts {lens}")
    st_ = (dataclasses.replace(dg.SHAPES["draft_a"], n_layers=1, vocab=2048, name="draft_a_1layer")
           if shape_name == "draft_a_1layer" else dg.SHAPES[shape_name])
    w = dg.make_weights(st_, 87, BF16_LM_SCALE)
    gm = api.Model(st_, w, max_rows=max_rows, max_pos=max(lens) + 64)
    B, gamma, V = len(lens), 3, st_.vocab
    prompts = [[int(t) for t in dg.make_prompt(87, b, n, V)] for b, n in enumerate(lens)]
    cand = H.dev(dg.make_prompt(88, 0, B * gamma, V).reshape(B, gamma).astype(np.int32))
    outs = []
    for opt in (0, 1):
        api.set_option("prefill_attn", opt)
        try:
            ctx = api.Context([n + 16 for n in lens])
            ctx.attach(gm)
            H.gpu_prefill(ctx, [gm], prompts)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            api.sd_verify(gm, ctx, None, B, gamma, 0.0, cand, None, None, na, nx, commit=False)
            ctx.sync()
            outs.append(gm.last_logits().cpu().numpy())
            ctx.close()
        finally:
            api.set_option("prefill_attn", 1)
    rel = np.abs(outs[0] - outs[1]).max() / np.abs(outs[0]).max()
    _say(f"  rel diff {rel:.2e}")
    assert np.isfinite(outs[1]).all() and rel < 5e-4
    gm.close()


@pytest.mark.parametrize("shape_name,max_rows", [("small_target_bf16", 512), ("small_draft_bf16", 384)])
def test_prefill_attention_at_every_prompt_length_matches_the_split_kernel(shape_name, max_rows):
    """Prompt lengths 17 to 208, eight consecutive ones per batch (four or three 16-row groups per sequence and
    forward): the last group of a prompt then ends at every offset inside a group and a 32-token tile, groups of a
    block end at different tiles, and sequences finish in different forwards.  Shared-tile kernel against the split
    kernel per group, verify logits of every sequence."""
    _say(f"{shape_name}: prefill attention at prompt lengths 17..208, workspace {max_rows}")
    st_ = dg.SHAPES[shape_name]
    w = dg.make_weights(st_, 89, BF16_LM_SCALE)
    gm = api.Model(st_, w, max_rows=max_rows, max_pos=256)
    B, gamma, V = 8, 3, st_.vocab
    cand = H.dev(dg.make_prompt(90, 0, B * gamma, V).reshape(B, gamma).astype(np.int32))
    worst = 0.0
    for n0 in range(17, 209, B):
        lens = list(range(n0, n0 + B))
        prompts = [[int(t) for t in dg.make_prompt(89, n, n, V)] for n in lens]
        outs = []
        for opt in (0, 1):
            api.set_option("prefill_attn", opt)
            try:
                ctx = api.Context([n + 16 for n in lens])
                ctx.attach(gm)
                H.gpu_prefill(ctx, [gm], prompts)
                na = torch.zeros(B, dtype=torch.int32, device="cuda")
                nx = torch.zeros(B, dtype=torch.int32, device="cuda")
                api.sd_verify(gm, ctx, None, B, gamma, 0.0, cand, None, None, na, nx, commit=False)
                ctx.sync()
                outs.append(gm.last_logits().cpu().numpy())
                ctx.close()
            finally:
                api.set_option("prefill_attn", 1)
        rel = np.abs(outs[0] - outs[1]).max() / np.abs(outs[0]).max()
        assert np.isfinite(outs[1]).all() and rel < 5e-4, (n0, rel)
        worst = max(worst, rel)
    _say(f"  worst rel diff {worst:.2e}")
    gm.close()


@pytest.mark.parametrize("shape_name,max_rows,lens", [("small_target_bf16", 112, [700, 45]), ("small_draft_bf16", 64, [1700]),
                                                      ("draft_a_1layer", 160, [333, 650, 16])])
def test_rope_and_cache_append_per_row_group_gives_the_bits_of_the_row_kernel(shape_name, max_rows, lens):
    """On the split attention path (prefill, long contexts) a bf16 model's RoPE + cache append runs one block per
    (head, group of up to 16 consecutive rows) with 16-byte stores; option rope_group = 0 brings back the block
    per row with its 2-byte stores.  Same fp32 sums in the same order and the same roundings: the verify logits
    after the prefill must be identical bit for bit.  Full groups at multiples of 16 (32-byte V runs), partial
    last groups, and a 1700-token context whose verify pass (4 rows per group) takes the split path as well."""
    import dataclasses
    _say(f"{shape_name}: RoPE + append per row group vs per row, workspace {max_rows}, prompts {lens}")
    st_ = (dataclasses.replace(dg.SHAPES["draft_a"], n_layers=1, vocab=2048, name="draft_a_1layer")
           if shape_name == "draft_a_1layer" else dg.SHAPES[shape_name])
    w = dg.make_weights(st_, 89, BF16_LM_SCALE)
    gm = api.Model(st_, w, max_rows=max_rows, max_pos=max(lens) + 64)
    B, gamma, V = len(lens), 3, st_.vocab
    prompts = [[int(t) for t in dg.make_prompt(89, b, n, V)] for b, n in enumerate(lens)]
    cand = H.dev(dg.make_prompt(90, 0, B * gamma, V).reshape(B, gamma).astype(np.int32))
    outs = []
    for opt in (0, 1):
        api.set_option("rope_group", opt)
        try:
            ctx = api.Context([n + 16 for n in lens])
            ctx.attach(gm)
            H.gpu_prefill(ctx, [gm], prompts)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            api.sd_verify(gm, ctx, None, B, gamma, 0.0, cand, None, None, na, nx, commit=False)
            ctx.sync()
            outs.append(gm.last_logits().cpu().numpy())
            ctx.close()
        finally:
            api.set_option("rope_group", 1)
    assert np.isfinite(outs[1]).all() and np.array_equal(outs[0], outs[1])
    gm.close()


@pytest.mark.parametrize("shape_name,keep", [("small_target_bf16", 37), ("small_draft_bf16", 101), ("draft_a_1layer", 16)])
def test_prefill_resumed_from_an_odd_cache_length_matches_the_prefill_from_zero(shape_name, keep):
    """A prompt is prefilled, its cache cut back to `keep` rows (not a multiple of 16 or 32 in two of the cases) and
    prefilled again: the row groups of the second pass start in the middle of a K / V tile, so the prefill attention
    masks inside its first tiles, the cache append takes its token-by-token path, and the new rows share tiles with
    old ones.  The rows written are the same as before, and the verify logits must agree with the untouched
    prefill's to rounding level."""
    import dataclasses
    _say(f"{shape_name}: prefill resumed from cache length {keep}")
    st_ = (dataclasses.replace(dg.SHAPES["draft_a"], n_layers=1, vocab=2048, name="draft_a_1layer")
           if shape_name == "draft_a_1layer" else dg.SHAPES[shape_name])
    w = dg.make_weights(st_, 93, BF16_LM_SCALE)
    gm = api.Model(st_, w, max_rows=96, max_pos=512)
    n, gamma, V = 333, 3, st_.vocab
    prompt = [int(t) for t in dg.make_prompt(93, 0, n, V)]
    cand = H.dev(dg.make_prompt(94, 0, gamma, V).reshape(1, gamma).astype(np.int32))
    outs = []
    for resume in (False, True):
        ctx = api.Context([n + 16])
        ctx.attach(gm)
        H.gpu_prefill(ctx, [gm], [prompt])
        if resume:
            ctx.truncate(gm, 0, keep)
            api.sd_prefill(gm, ctx, None, 1, n - 1 - keep)
        nt, kv = ctx.sync(gm)
        assert list(nt) == [n] and list(kv) == [n - 1]
        na = torch.zeros(1, dtype=torch.int32, device="cuda")
        nx = torch.zeros(1, dtype=torch.int32, device="cuda")
        api.sd_verify(gm, ctx, None, 1, gamma, 0.0, cand, None, None, na, nx, commit=False)
        ctx.sync()
        outs.append(gm.last_logits().cpu().numpy())
        ctx.close()
    rel = np.abs(outs[0] - outs[1]).max() / np.abs(outs[0]).max()
    _say(f"  rel diff {rel:.2e}")
    assert np.isfinite(outs[1]).all() and rel < 5e-4
    gm.close()


@pytest.mark.parametrize("shape_name", ["small_target_bf16", "small_draft_bf16", "tiny_target"])
def test_the_same_call_twice_gives_the_same_bits(shape_name):
    """Prefill in row groups, a sampled draft call and a verify pass of a ragged batch, run twice from fresh
    contexts: logits, q, candidates and decisions must be bit-identical (no result depends on the order in which
    blocks or atomics happen to finish)."""
    _say(f"{shape_name}: repeatability")
    st_ = dg.SHAPES[shape_name]
    w = dg.make_weights(st_, 95, BF16_LM_SCALE if st_.dtype == dg.BF16 else 20.0)
    gm = api.Model(st_, w, max_rows=96, max_pos=512)
    B, gamma, V, T = 5, 4, st_.vocab, 0.8
    lens = [300, 33, 170, 5, 64]
    prompts = [[int(t) for t in dg.make_prompt(95, b, n, V)] for b, n in enumerate(lens)]
    ud = H.dev(np.stack([dg.make_uniforms(95, dg.DRAFT_STREAM, b, 0, gamma) for b in range(B)]))
    uv = H.dev(np.stack([dg.make_uniforms(95, dg.VERIFY_STREAM, b, 0, gamma + 1) for b in range(B)]))
    runs = []
    for rep in range(2):
        ctx = api.Context([n + 16 for n in lens])
        ctx.attach(gm)
        H.gpu_prefill(ctx, [gm], prompts)
        cand = torch.full((B, gamma), -1, dtype=torch.int32, device="cuda")
        q = torch.zeros((B, gamma, V), dtype=torch.float32, device="cuda")
        api.sd_draft(gm, ctx, None, B, gamma, T, ud, cand, q)
        ctx.sync()
        for b in range(B):
            ctx.truncate(gm, b, lens[b] - 1)
        na = torch.zeros(B, dtype=torch.int32, device="cuda")
        nx = torch.zeros(B, dtype=torch.int32, device="cuda")
        api.sd_verify(gm, ctx, None, B, gamma, T, cand, q, uv, na, nx, commit=True)
        nt, kv = ctx.sync(gm)
        runs.append((cand.cpu().numpy(), q.cpu().numpy(), gm.last_logits().cpu().numpy(), na.cpu().numpy(),
                     nx.cpu().numpy(), np.array(nt), np.array(kv)))
        ctx.close()
    for a, b in zip(runs[0], runs[1]):
        assert np.array_equal(a, b)
    assert np.isfinite(runs[0][2]).all()
    gm.close()


def test_small_bf16_ragged_batch_of_tiny_and_very_long_contexts():
    """One batch whose contexts run from 3 to 4000 tokens (3, 9, 33, 40, 700, 1500, 2049, 4000): one to 126 K / V
    tiles per sequence in the same attention launch, which therefore takes the split-KV kernel with most splits of
    the short sequences empty; draft and verify compared with the oracle step by step along each sequence's own
    trajectory, T = 1."""
    _say("small bf16: ragged batch, contexts 3..4000")
    st_, sd_ = dg.SHAPES["small_target_bf16"], dg.SHAPES["small_draft_bf16"]
    seed, gamma = 97, 4
    lens = [3, 4000, 40, 1500, 700, 9, 2049, 33]
    V = st_.vocab
    wt, wd = dg.make_weights(st_, seed, BF16_LM_SCALE), dg.make_weights(sd_, seed + 1, BF16_LM_SCALE)
    ot, od = oracle.OracleModel(st_, wt), oracle.OracleModel(sd_, wd)
    gt = api.Model(st_, wt, max_rows=64, max_pos=4200)
    gd = api.Model(sd_, wd, max_rows=64, max_pos=4200)
    prompts = [[int(t) for t in dg.make_prompt(seed, b, n, V)] for b, n in enumerate(lens)]
    n, flagged = H.batched_teacher_forced(gt, gd, ot, od, prompts, gamma, 1.0, 24, seed, dg.BF16, None)
    _say(f"  steps={n} flagged={flagged}")
    assert n >= 5 and flagged <= H.flag_cap(n * len(lens))
    gt.close()
    gd.close()


def test_gamma_zero_is_autoregressive_decoding(tiny_pair):
    _say("gamma = 0")
    prompt = dg.make_prompt(11, 2, 12, TINY_T.vocab)
    ar, _ = oracle.ar_generate(tiny_pair.ot.new_seq(64), prompt, 0.0, 16, H.uf(1, dg.VERIFY_STREAM))
    ctx = api.Context([64])
    ctx.attach(tiny_pair.gt)
    H.gpu_prefill(ctx, [tiny_pair.gt], [list(prompt)])
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    nx = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(16):
        api.sd_verify(tiny_pair.gt, ctx, None, 1, 0, 0.0, None, None, None, na, nx, commit=True)
    ctx.sync()
    assert list(ctx.get_tokens(0)[12:]) == ar
    ctx.close()


def test_batched_sequences_with_seq_ids(tiny_pair):
    """Three ragged sequences in one context; calls select subsets through seq_ids.
    Every sequence must behave exactly as it does alone."""
    _say("batched seq_ids")
    gamma, T = 3, 1.0
    prompts = [dg.make_prompt(51, i, n, TINY_T.vocab) for i, n in enumerate((5, 23, 14))]
    trajs = [H.oracle_trajectory(tiny_pair, p, gamma, T, 12, seed=51, seq=i, keep_logits=False)
             for i, p in enumerate(prompts)]
    ctx = api.Context([t[2] for t in trajs])
    ctx.attach(tiny_pair.gt)
    ctx.attach(tiny_pair.gd)
    H.gpu_prefill(ctx, [tiny_pair.gt, tiny_pair.gd], [list(p) for p in prompts])
    V = TINY_T.vocab
    order = [2, 0, 1]                 # rows of the call are a permutation of the context's sequences
    ids = H.dev(np.array(order, np.int32))
    cand = torch.zeros((3, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((3, gamma, V), dtype=torch.float32, device="cuda")
    na = torch.zeros(3, dtype=torch.int32, device="cuda")
    nx = torch.zeros(3, dtype=torch.int32, device="cuda")
    n_steps = min(len(t[1]) for t in trajs)
    for k in range(n_steps):
        ud = H.dev(np.stack([trajs[b][1][k].u_draft for b in order]))
        uv = H.dev(np.stack([trajs[b][1][k].u_verify for b in order]))
        api.sd_draft(tiny_pair.gd, ctx, ids, 3, gamma, T, ud, cand, q)
        ref_c = np.stack([trajs[b][1][k].cand for b in order])
        ref_q = np.stack([trajs[b][1][k].q for b in order])
        assert np.array_equal(cand.cpu().numpy(), ref_c), k
        assert np.abs(q.cpu().numpy() - ref_q).max() < 1e-5
        api.sd_verify(tiny_pair.gt, ctx, ids, 3, gamma, T, H.dev(ref_c), H.dev(ref_q), uv, na, nx, commit=True)
        assert list(na.cpu().numpy()) == [trajs[b][1][k].n_acc for b in order], k
        assert list(nx.cpu().numpy()) == [trajs[b][1][k].next_token for b in order], k
    nt, _ = ctx.sync()
    for b in range(3):
        assert nt[b] == len(prompts[b]) + sum(s.n_acc + 1 for s in trajs[b][1][:n_steps])
    ctx.close()


@pytest.mark.parametrize("rho,vocab", [(0.0, 32000), (0.5, 32000), (0.9, 32000), (0.5, 50000)])
def test_verify_tail_full_vocabulary_synthetic_q(rho, vocab):
    """Config-5 style stress of the fused softmax/accept/residual/resample kernel at the
    real vocabulary (32000) in fp32, where logits agree to ~1e-7 and every decision must
    match the oracle to the 1e-5 base threshold: batch of 8 ragged sequences, gamma = 8,
    draft distributions q = softmax(rho * target logits + (1 - rho) * 4 * N(0,1)), candidates
    drawn from q, built position by position with the oracle only.  A vocabulary of 50000 does
    not fit the register-resident row kernels (32768 entries) and takes the strided ones, in the
    verify tail and in the draft's sampling (checked here too, with the model drafting for itself)."""
    _say(f"verify tail, V={vocab}, rho={rho}")
    shape = dg.ModelShape("wide_vocab_fp32", 1, 64, 1, 64, 128, vocab, dg.FP32)
    w = dg.make_weights(shape, 71, lm_head_scale=20.0)   # logit std 0.02*20*8 = 3.2
    om = oracle.OracleModel(shape, w)
    gm = api.Model(shape, w, max_rows=72, max_pos=128)
    B, gamma, T, V = 8, 8, 1.0, shape.vocab
    if vocab > 32768:   # the draft's sampling kernel on the same wide rows
        pr = [dg.make_prompt(72, b, 5 + 7 * b, V) for b in range(3)]
        c2 = api.Context([64] * 3)
        c2.attach(gm)
        H.gpu_prefill(c2, [gm], [list(p) for p in pr])
        ud = np.stack([dg.make_uniforms(72, dg.DRAFT_STREAM, b, 0, 4) for b in range(3)])
        cand_g = torch.zeros((3, 4), dtype=torch.int32, device="cuda")
        q_g = torch.zeros((3, 4, V), dtype=torch.float32, device="cuda")
        api.sd_draft(gm, c2, None, 3, 4, T, H.dev(ud), cand_g, q_g)
        for b in range(3):
            seq = om.new_seq(64)
            oracle.prefill(seq, [int(t) for t in pr[b]])
            r_c, r_q, mg = seq.draft([int(t) for t in pr[b]], 4, T, ud[b])
            got = cand_g[b].cpu().numpy()
            if not np.array_equal(got, r_c):   # only a draw within 1e-5 of a CDF step may differ
                k = int(np.argmax(got != r_c))
                assert mg[k] < 1e-5, (b, got, r_c, mg)
            else:
                assert np.abs(q_g[b].cpu().numpy() - r_q).max() < 1e-6
        c2.close()
    lens = dg.make_prompt_lengths(71, B, 3, 40)
    prompts = [dg.make_prompt(71, b, int(lens[b]), V) for b in range(B)]
    cands, qs, us, refs = [], [], [], []
    for b in range(B):
        seq = om.new_seq(64)
        ctx_t = [int(t) for t in prompts[b]]
        oracle.prefill(seq, ctx_t)
        ud = dg.make_uniforms(71, dg.DRAFT_STREAM, b, 0, gamma)
        cand, q = [], np.zeros((gamma, V), np.float32)
        for i in range(gamma):
            lg = seq.forward([ctx_t[-1]] + cand)[-1]
            seq.truncate(len(ctx_t) - 1)
            z = rho * lg + (1.0 - rho) * 4.0 * dg.make_logit_noise(71, b, i, V)
            q[i] = oracle.softmax_T(z.astype(np.float32), 1.0)
            cand.append(oracle.sample_cdf(q[i].astype(np.float64), float(ud[i]))[0])
        uv = dg.make_uniforms(71, dg.VERIFY_STREAM, b, 0, gamma + 1)
        refs.append(seq.verify(ctx_t, gamma, T, cand, q, uv, want_logits=True))
        cands.append(cand)
        qs.append(q)
        us.append(uv)
    ctx = api.Context([64] * B)
    ctx.attach(gm)
    H.gpu_prefill(ctx, [gm], [list(p) for p in prompts])
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    api.sd_verify(gm, ctx, None, B, gamma, T, H.dev(np.array(cands, np.int32)), H.dev(np.stack(qs)),
                  H.dev(np.stack(us)), na, nx, commit=True)
    lg = gm.last_logits().cpu().numpy().reshape(B, gamma + 1, V)
    na, nx = na.cpu().numpy(), nx.cpu().numpy()
    accs = []
    for b in range(B):
        r_na, r_nx, mg, r_lg = refs[b]
        assert np.abs(lg[b] - r_lg).max() / np.abs(r_lg).max() < 1e-4
        if (na[b], nx[b]) != (r_na, r_nx):
            assert mg[:min(r_na, na[b]) + 1].min() < 1e-5 or mg[gamma] < 1e-5, (b, na[b], nx[b], r_na, r_nx, mg)
        accs.append(r_na)
    _say(f"  n_acc per sequence: {accs}")
    nt, kv = ctx.sync(gm)
    for b in range(B):   # ragged rollback: each sequence advanced by its own n_acc + 1
        assert nt[b] == lens[b] + na[b] + 1 and kv[b] == nt[b] - 1
    if rho == 0.9:
        assert max(accs) >= 2
    ctx.close()
    gm.close()


def test_route_matches_oracle():
    W, b = dg.make_router(7)
    e = dg.make_prompt_embeddings(7, 32)
    out = torch.zeros(32, dtype=torch.int32, device="cuda")
    api.sd_route(H.dev(W), H.dev(b), H.dev(e), out)
    ref = oracle.route(W, b, e)
    assert np.array_equal(out.cpu().numpy(), ref) and len(set(ref)) == 4


def test_capacity_and_state_errors_are_reported_not_faulted(tiny_pair):
    _say("error paths")
    ctx = api.Context([16])
    ctx.attach(tiny_pair.gt)
    with pytest.raises(api.SdError) as ei:
        ctx.set_tokens([list(range(100))])
    assert ei.value.code == api.SD_ECAP
    H.gpu_prefill(ctx, [tiny_pair.gt], [list(range(10))])
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    nx = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(api.SdError) as ei:
        api.sd_verify(tiny_pair.gt, ctx, None, 1, 16, 0.0, na, None, None, na, nx)
    assert ei.value.code == api.SD_ECAP
    with pytest.raises(api.SdError) as ei:
        api.sd_verify(tiny_pair.gd, ctx, None, 1, 2, 0.0, na, None, None, na, nx)  # draft was never attached
    assert ei.value.code == api.SD_EINVAL
    cand = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    for bad_n in (0, 2):   # an empty batch, and more sequences than the context holds
        with pytest.raises(api.SdError) as ei:
            api.sd_verify(tiny_pair.gt, ctx, None, bad_n, 4, 0.0, cand, None, None, na, nx)
        assert ei.value.code == api.SD_EINVAL
    # run the sequence into its capacity: the kernels refuse the rows and raise the flag
    for _ in range(70):
        api.sd_verify(tiny_pair.gt, ctx, None, 1, 4, 0.0, cand, None, None, na, nx, commit=True)
    with pytest.raises(api.SdError) as ei:
        ctx.sync()
    assert ei.value.code == api.SD_ESTATE and "capacity" in str(ei.value)
    nt, _ = ctx.sync()
    assert nt[0] <= 64
    ctx.close()


@pytest.mark.parametrize("shape_name,tol", [("tiny_draft", 1e-4), ("small_target_bf16", 2e-2)])
def test_lora_adapters_chosen_per_sequence_match_oracle(shape_name, tol):
    """Section 2.3's drafts are LoRA fine-tunes of one base model: a batch whose sequences use different
    adapters (and one none) runs as ONE forward of the base with per-sequence low-rank updates on q, k, v, o.
    Prefill, a draft call (candidates and q) and a verify-style pass (logits) are compared per sequence with
    the oracle run on that sequence alone with its adapter.  fp32 takes the reference kernels (updates
    added in place), bf16 the MFMA kernels (update = one more split-K slab)."""
    _say(f"LoRA adapters per sequence, {shape_name}")
    st_ = dg.SHAPES[shape_name]
    bf = st_.dtype == dg.BF16
    w = dg.make_weights(st_, 95, BF16_LM_SCALE if bf else 20.0)
    lora = dg.make_lora(st_, 96, n_adapters=3, rank=8, std_a=0.05, std_b=0.05)
    scale, gamma, V = 2.0, 4, st_.vocab
    om = oracle.OracleModel(st_, w)
    om.set_lora(lora, scale)
    gm = api.Model(st_, w, max_rows=32, max_pos=256)
    gm.set_lora(lora, scale)
    adapters = [0, -1, 2, 1]
    lens = [12, 33, 7, 20]
    B = len(lens)
    prompts = [[int(t) for t in dg.make_prompt(95, b, n, V)] for b, n in enumerate(lens)]
    ctx = api.Context([n + 32 for n in lens])
    ctx.attach(gm)
    ctx.set_adapters(gm, adapters)
    H.gpu_prefill(ctx, [gm], prompts)
    # draft call: the model drafts for itself, sampled
    T = 1.0
    ud = np.stack([dg.make_uniforms(95, dg.DRAFT_STREAM, b, 0, gamma) for b in range(B)])
    cand = torch.zeros((B, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((B, gamma, V), dtype=torch.float32, device="cuda")
    api.sd_draft(gm, ctx, None, B, gamma, T, H.dev(ud), cand, q)
    cg, qg = cand.cpu().numpy(), q.cpu().numpy()
    base_differs = 0
    for b in range(B):
        seq = om.new_seq(lens[b] + 32, adapters[b])
        oracle.prefill(seq, prompts[b])
        r_c, r_q, mg = seq.draft(prompts[b], gamma, T, ud[b])
        k = 0
        while k < gamma and cg[b][k] == r_c[k]:
            assert np.abs(qg[b][k] - r_q[k]).max() < (2e-3 if bf else 1e-5), (b, k)
            k += 1
        if k < gamma:   # a differing token must be a low-margin draw
            assert mg[k] < (5e-2 if bf else 1e-4), (b, k, cg[b], r_c, mg)
        if adapters[b] >= 0:   # and the adapter must matter: the base model drafts another distribution
            sb = oracle.OracleModel(st_, w).new_seq(lens[b] + 32)
            oracle.prefill(sb, prompts[b])
            _, b_q, _ = sb.draft(prompts[b], 1, T, ud[b][:1])
            base_differs += int(np.abs(b_q[0] - r_q[0]).max() > 10 * (2e-3 if bf else 1e-5))
    assert base_differs >= 2
    ctx.sync()
    ctx.close()
    gm.close()


def test_online_path_classifier_routes_to_adapters_of_one_base_draft():
    """The whole online path in its shared-base form (Sections 2.3, 2.4): the prompt classifier labels each
    prompt from its token ids, the label names the low-rank adapter of the one base draft (the last class
    means the plain base), ALL sequences draft in one batch, the target verifies them in one call.  Every
    sequence must behave as it does alone in the oracle with the adapter the oracle's classifier picks."""
    from oracle import mamba
    _say("online path: classifier -> adapters -> one draft batch -> verify")
    gamma, T, B, n_tok, seed = 4, 0.8, 9, 14, 97
    st_ = dg.SHAPES["small_target_bf16"]
    V = st_.vocab
    sd_ = dg.ModelShape("d_shared", 2, 128, 2, 64, 384, V, dg.BF16)
    cs = dataclasses.replace(dg.CLASSIFIER_TINY, name="classifier_online", vocab=V, n_classes=4)
    wt = dg.make_weights(st_, seed, BF16_LM_SCALE)
    wd = dg.make_weights(sd_, seed + 1, BF16_LM_SCALE)
    lora = dg.make_lora(sd_, seed + 2, n_adapters=3, rank=8, std_a=0.05, std_b=0.05)
    wc = dg.make_classifier(cs, 103)     # a seed whose labels cover all four classes with clear margins
    lens = dg.make_prompt_lengths(seed, B, 16, 90)
    prompts = [[int(t) for t in dg.make_prompt(seed, b, int(lens[b]), V)] for b in range(B)]
    # routing on both sides
    max_len = int(lens.max())
    tok = np.zeros((B, max_len), np.int32)
    for b in range(B):
        tok[b, :lens[b]] = prompts[b]
    ids_g = torch.zeros(B, dtype=torch.int32, device="cuda")
    cls = api.Classifier(cs, wc)
    cls.route(H.dev(tok), H.dev(lens.astype(np.int32)), ids_g)
    labels = [mamba.classify(wc, prompts[b])[1] for b in range(B)]
    assert ids_g.cpu().numpy().tolist() == labels and len(set(labels)) == 4, labels
    cls.close()
    adapters = [l if l < 3 else -1 for l in labels]
    ot, od = oracle.OracleModel(st_, wt), oracle.OracleModel(sd_, wd)
    od.set_lora(lora, 2.0)
    gt = api.Model(st_, wt, max_rows=B * (gamma + 1), max_pos=256)
    gd = api.Model(sd_, wd, max_rows=2 * B, max_pos=256)
    gd.set_lora(lora, 2.0)
    n_steps, flagged = H.batched_teacher_forced(gt, gd, ot, od, prompts, gamma, T, n_tok, seed, dg.BF16, adapters)
    _say(f"  labels={labels} steps={n_steps} flagged={flagged}")
    assert n_steps >= 4 and flagged <= 2
    gt.close()
    gd.close()


def test_random_shapes_single_sequence_and_ragged_batches():
    """Seeded sweep over legal model shapes the fixed configurations do not visit (head widths 16..128, one to
    four heads, FFN and vocabulary sizes that are and are not multiples of the kernels' tile widths, fp32 and
    bf16, gamma 1..8, greedy and sampled): one sequence teacher-forced, then a ragged batch of 2..7 sequences
    drafted and verified in single calls.  Shapes outside the MFMA kernels' domain take the reference
    kernels matrix by matrix, so this also covers models that mix both."""
    rng = np.random.default_rng(20250508)
    flagged = steps = 0
    worst = {dg.BF16: 0.0, dg.FP32: 0.0}
    for it in range(36):
        dt = dg.BF16 if rng.integers(0, 2) else dg.FP32
        V = int(rng.integers(40, 700)) * 4
        if it % 2:      # widths the MFMA kernels take (multiples of 128), FFN a multiple of 128 or only of 16
            hd = int(rng.choice([64, 128]))
            h_t, h_d = int(rng.integers(1, 4)) * (128 // hd), int(rng.integers(1, 3)) * (128 // hd)
            f_t, f_d = int(rng.integers(1, 8)) * int(rng.choice([128, 16])), int(rng.integers(1, 6)) * 128
        else:
            hd = int(rng.choice([16, 32, 64, 128]))
            h_t, h_d = int(rng.integers(1, 5)), int(rng.integers(1, 3))
            f_t, f_d = int(rng.integers(3, 60)) * 16, int(rng.integers(3, 40)) * 16
        st_ = dg.ModelShape("rt", int(rng.integers(1, 4)), h_t * hd, h_t, hd, f_t, V, dt)
        sd_ = dg.ModelShape("rd", int(rng.integers(1, 3)), h_d * hd, h_d, hd, f_d, V, dt)
        gamma, T = int(rng.integers(1, 9)), float(rng.choice([0.0, 0.7, 1.0]))
        seed, plen, B = int(rng.integers(1, 10000)), int(rng.integers(2, 150)), int(rng.integers(2, 8))
        _say(f"random shape {it}: {st_} / {sd_} gamma={gamma} T={T} seed={seed} plen={plen} B={B}")
        pair = H.Pair(st_, sd_, seed=seed, lm_scale=BF16_LM_SCALE if dt == dg.BF16 else 20.0,
                      max_rows=max(32, B * (gamma + 1)))
        s = H.teacher_forced_parity(pair, [int(t) for t in dg.make_prompt(seed, 0, plen, V)], gamma, T, 12, seed)
        flagged, steps = flagged + s.flagged, steps + s.steps
        worst[dt] = max(worst[dt], s.max_logit_rel)
        lens = dg.make_prompt_lengths(seed, B, 2, 100)
        prompts = [[int(t) for t in dg.make_prompt(seed, b, int(lens[b]), V)] for b in range(B)]
        n, f = H.batched_teacher_forced(pair.gt, pair.gd, pair.ot, pair.od, prompts, gamma, T, 8, seed, dt)
        flagged, steps = flagged + f, steps + n * B
        pair.close()
    _say(f"  steps={steps} flagged={flagged} worst logit error bf16 {worst[dg.BF16]:.2e} fp32 {worst[dg.FP32]:.2e}")
    assert worst[dg.BF16] <= 2e-2 and worst[dg.FP32] <= 1e-4
    assert flagged <= H.flag_cap(steps)


def test_draft_groups_on_separate_streams_match_sequential_calls():
    """The drafts of a routed batch are independent models with workspaces of their own, so their sd_draft
    calls may run on different streams at the same time (all at the default priority).  Four drafts of
    different shapes, two sequences each: candidates and q from the concurrent calls must equal, bit for
    bit, those of the same calls issued one after the other."""
    _say("draft groups on four streams")
    gamma, T, B, seed = 5, 0.7, 8, 93
    V = 2048
    dshapes = [dg.ModelShape("d_a", 1, 128, 2, 64, 384, V, dg.BF16), dg.ModelShape("d_b", 2, 128, 2, 64, 256, V, dg.BF16),
               dg.ModelShape("d_c", 1, 256, 4, 64, 512, V, dg.BF16), dg.ModelShape("d_d", 1, 64, 1, 64, 128, V, dg.BF16)]
    gds = [api.Model(sh, dg.make_weights(sh, seed + i, BF16_LM_SCALE), max_rows=16, max_pos=256) for i, sh in enumerate(dshapes)]
    groups = [[g, g + 4] for g in range(4)]
    lens = dg.make_prompt_lengths(seed, B, 8, 100)
    prompts = [[int(t) for t in dg.make_prompt(seed, b, int(lens[b]), V)] for b in range(B)]
    ctx = api.Context([int(l) + 32 for l in lens])
    for gd in gds:
        ctx.attach(gd)
    ctx.set_tokens(prompts)
    gid = [H.dev(np.array(g, np.int32)) for g in groups]
    for g in range(4):
        api.sd_prefill(gds[g], ctx, gid[g], 2, max(int(lens[b]) for b in groups[g]) - 1)
    ud = [H.dev(np.stack([dg.make_uniforms(seed, dg.DRAFT_STREAM, b, 0, gamma) for b in groups[g]])) for g in range(4)]

    def fresh():
        return ([torch.zeros((2, gamma), dtype=torch.int32, device="cuda") for _ in range(4)],
                [torch.zeros((2, gamma, V), dtype=torch.float32, device="cuda") for _ in range(4)])

    def rewind():   # back to the state after prefill: each draft's cache length = tokens - 1
        torch.cuda.synchronize()
        for g in range(4):
            for b in groups[g]:
                ctx.truncate(gds[g], b, int(lens[b]) - 1)

    cand_a, q_a = fresh()
    for g in range(4):
        api.sd_draft(gds[g], ctx, gid[g], 2, gamma, T, ud[g], cand_a[g], q_a[g])
    rewind()
    cand_b, q_b = fresh()
    main = torch.cuda.current_stream()
    streams = [torch.cuda.Stream() for _ in range(4)]
    for g in range(4):
        streams[g].wait_stream(main)
        with torch.cuda.stream(streams[g]):
            api.sd_draft(gds[g], ctx, gid[g], 2, gamma, T, ud[g], cand_b[g], q_b[g])
    for g in range(4):
        main.wait_stream(streams[g])
    torch.cuda.synchronize()
    for g in range(4):
        assert torch.equal(cand_a[g], cand_b[g]) and torch.equal(q_a[g], q_b[g]), g
        assert int(cand_a[g].min()) >= 0 and float(q_a[g].sum(-1).min()) > 0.999
    ctx.sync()
    ctx.close()
    for gd in gds:
        gd.close()


def test_config3_routed_heterogeneous_drafts_small():
    """BASELINE config 3's structure at small widths: a batch of ragged prompts, each routed by the
    linear classifier to one of four drafts of different shapes; every draft decodes its group
    (seq_ids), the target verifies all sequences in one call (T = 0.7, gamma = 5).  Every
    sequence must behave exactly as it does alone in the oracle."""
    _say("config 3 (small): routed heterogeneous drafts")
    gamma, T, B, n_tok, seed = 5, 0.7, 10, 18, 91
    st_ = dg.SHAPES["small_target_bf16"]
    V = st_.vocab
    dshapes = [dg.ModelShape("d_a", 1, 128, 2, 64, 384, V, dg.BF16), dg.ModelShape("d_b", 2, 128, 2, 64, 256, V, dg.BF16),
               dg.ModelShape("d_c", 1, 256, 4, 64, 512, V, dg.BF16), dg.ModelShape("d_d", 1, 64, 1, 64, 128, V, dg.BF16)]
    wt = dg.make_weights(st_, seed, BF16_LM_SCALE)
    wds = [dg.make_weights(sh, seed + 1 + i, BF16_LM_SCALE) for i, sh in enumerate(dshapes)]
    ot = oracle.OracleModel(st_, wt)
    ods = [oracle.OracleModel(sh, w) for sh, w in zip(dshapes, wds)]
    gt = api.Model(st_, wt, max_rows=B * (gamma + 1), max_pos=256)
    gds = [api.Model(sh, w, max_rows=2 * B, max_pos=256) for sh, w in zip(dshapes, wds)]
    # routing: GPU classifier vs oracle
    Wr, br = dg.make_router(seed)
    emb = dg.make_prompt_embeddings(seed, B)
    ids_g = torch.zeros(B, dtype=torch.int32, device="cuda")
    api.sd_route(H.dev(Wr), H.dev(br), H.dev(emb), ids_g)
    route = oracle.route(Wr, br, emb)
    assert np.array_equal(ids_g.cpu().numpy(), route)
    groups = [[b for b in range(B) if route[b] == g] for g in range(4)]
    assert sum(1 for g in groups if g) >= 3, groups
    lens = dg.make_prompt_lengths(seed, B, 16, 120)
    prompts = [[int(t) for t in dg.make_prompt(seed, b, int(lens[b]), V)] for b in range(B)]
    # oracle: every sequence on its own
    trajs = []
    for b in range(B):
        cap = len(prompts[b]) + n_tok + 2 * gamma + 4
        toks, steps = oracle.sd_generate(ot.new_seq(cap), ods[route[b]].new_seq(cap), prompts[b], gamma, T, n_tok,
                                         H.uf(seed, dg.DRAFT_STREAM, b), H.uf(seed, dg.VERIFY_STREAM, b),
                                         keep_logits=True)
        trajs.append(steps)
    n_steps = min(len(t) for t in trajs)
    ctx = api.Context([len(p) + (n_steps + 1) * (gamma + 1) + 8 for p in prompts])
    ctx.attach(gt)
    for gd in gds:
        ctx.attach(gd)
    ctx.set_tokens(prompts)
    api.sd_prefill(gt, ctx, None, B, max(len(p) for p in prompts) - 1)
    gid = [H.dev(np.array(g, np.int32)) if g else None for g in groups]
    for g in range(4):
        if groups[g]:
            api.sd_prefill(gds[g], ctx, gid[g], len(groups[g]), max(len(prompts[b]) for b in groups[g]) - 1)
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    flagged = 0
    for k in range(n_steps):
        refeed = []
        for g in range(4):
            if not groups[g]:
                continue
            ng = len(groups[g])
            ud = H.dev(np.stack([trajs[b][k].u_draft for b in groups[g]]))
            cand = torch.zeros((ng, gamma), dtype=torch.int32, device="cuda")
            q = torch.zeros((ng, gamma, V), dtype=torch.float32, device="cuda")
            api.sd_draft(gds[g], ctx, gid[g], ng, gamma, T, ud, cand, q)
            cg, qg = cand.cpu().numpy(), q.cpu().numpy()
            for j, b in enumerate(groups[g]):
                f, first_bad, _ = H.check_draft_step(trajs[b][k], cg[j], qg[j], T, dg.BF16, V)
                flagged += int(f)
                if first_bad is not None:   # that draft cache holds rows of other candidates from here on
                    refeed.append((g, b, trajs[b][k].n_ctx - 1 + first_bad))
        cand_all = H.dev(np.stack([trajs[b][k].cand for b in range(B)]).astype(np.int32))
        q_all = H.dev(np.stack([trajs[b][k].q for b in range(B)]))
        uv = H.dev(np.stack([trajs[b][k].u_verify for b in range(B)]))
        api.sd_verify(gt, ctx, None, B, gamma, T, cand_all, q_all, uv, na, nx, commit=False)
        lg = gt.last_logits().cpu().numpy().reshape(B, gamma + 1, V)
        na_h, nx_h = na.cpu().numpy(), nx.cpu().numpy()
        for b in range(B):
            f, _ = H.check_verify_step(trajs[b][k], int(na_h[b]), int(nx_h[b]), lg[b], T, dg.BF16, V)
            flagged += int(f)
        api.sd_commit(ctx, None, B, gamma, cand_all, H.dev(np.array([trajs[b][k].n_acc for b in range(B)], np.int32)),
                      H.dev(np.array([trajs[b][k].next_token for b in range(B)], np.int32)))
        for g, b, keep in refeed:   # roll that sequence's draft cache back and re-feed the committed tokens
            torch.cuda.synchronize()
            ctx.truncate(gds[g], b, keep)
            api.sd_prefill(gds[g], ctx, H.dev(np.array([b], np.int32)), 1, gamma + 2)
    nt, kv = ctx.sync(gt)
    for b in range(B):
        assert nt[b] == len(prompts[b]) + sum(s.n_acc + 1 for s in trajs[b][:n_steps]) and kv[b] == nt[b] - 1
    _say(f"  groups={[len(g) for g in groups]} steps={n_steps} flagged={flagged} "
         f"n_acc={[trajs[b][0].n_acc for b in range(B)]}")
    assert flagged <= 2
    ctx.close()
    gt.close()
    for gd in gds:
        gd.close()
