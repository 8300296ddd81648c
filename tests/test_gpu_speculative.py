"""GPU parity of the speculative anchor route of ttf_compress: the anchor rule is first guessed from
256 channels, the search runs against a trusted guess while adding up exact frame sums on the side,
and the exact rule then confirms the guess or has the clip searched again.  Whatever happens on the
way, every output must equal the oracle's.  The cases force the route on small inputs
(ttf_set_speculation(1)) and cover: confirmed guesses on every kernel layout the route has,
guesses that are trusted but wrong (second search), clips without a clear guess (two-pass
fallback), and all three kinds in one batch.  Which kind a clip is, is recomputed here in NumPy
from the rule the header documents, so that each case is known to exercise its branch."""
import numpy as np
import pytest

from workloads import CONFIGS, make_clip_batch
from workloads.ttf_gen import bf16_bits_to_f32

from helpers import compare_with_oracle, run_gpu

pytestmark = pytest.mark.gpu

TRUST_GAP = 0.1          # include/ttf.h: a guess is trusted when it beats the runner-up by this much


def guess_channels(C):
    """The 256 channels the guess looks at: four runs of 64, run j from (2j+1)*C/8 rounded down to 64."""
    return np.concatenate([np.arange(s, s + 64) for s in (((2 * j + 1) * C // 8) // 64 * 64 for j in range(4))])


def anchor_scores(fs):
    g = fs.sum(0)
    return (fs @ g) / (np.sqrt((fs * fs).sum(1)) * np.sqrt(g @ g))


def guess_of(x_clip_bits):
    """(guessed frame, gap to the runner-up) of one clip [F,H,W,C] of bf16 bit patterns."""
    F, C = x_clip_bits.shape[0], x_clip_bits.shape[-1]
    x = bf16_bits_to_f32(x_clip_bits).reshape(F, -1, C)[:, :, guess_channels(C)]
    sc = anchor_scores(x.sum(1, dtype=np.float64))
    order = np.argsort(-sc, kind="stable")
    return int(order[0]), float(sc[order[0]] - sc[order[1]])


def _check(batch, cfg, expect):
    """Enforce margins, classify every clip, run both routes, compare with the oracle."""
    from oracle import margins
    res = margins.enforce_margins(batch, cfg.r, cfg.t, want_tokens=False)
    kinds = []
    for b in range(cfg.B):
        a, gap = guess_of(batch.x[b])
        assert abs(gap - TRUST_GAP) > 0.02, "guess too close to the trust threshold for a robust test"
        kinds.append("fallback" if gap < TRUST_GAP else ("confirmed" if a == res.anchor_index[b] else "refuted"))
    assert kinds == list(expect), kinds
    for mode in (1, -1):
        _, out = run_gpu(batch.x, cfg.r, cfg.t[0], speculation=mode)
        compare_with_oracle(batch.x, out, res)
    return res


SHAPES = [
    # B, F,  H,  W,  C,    r
    (3, 6, 16, 16, 1024, 1),     # 4 waves x 2 K-steps per pass
    (2, 9, 8, 32, 1024, 1),      # 32-wide grid
    (2, 6, 16, 16, 1152, 1),     # 36 K-steps: one K-step per pass
    (1, 7, 16, 16, 2048, 0),     # 1x1 window
    (2, 6, 16, 16, 1024, 2),     # 5x5 window on a 16-wide grid
    (1, 9, 4, 32, 1024, 0),      # two keep words per frame on a 32-wide grid
    (2, 8, 16, 32, 1024, 2),     # 5x5 window on a 32-wide grid (few workgroups: the plain kernel)
    (1, 2, 16, 16, 1024, 1),     # one source frame
    (2, 33, 16, 16, 1024, 1),    # 33 frames: nine groups of four, the last with one frame
    (40, 13, 16, 16, 1024, 1),   # enough workgroups for the one-wave layout (6144 and more)
    (2, 18, 64, 32, 1024, 2),    # 5x5 window on a large 32-wide input: the kernel with anchors shared through LDS
    (1, 21, 128, 32, 1024, 2),   # the same kernel, 21 frames: five full groups of four and one frame
    # grids that are not exactly 16 or 32 wide, or whose height leaves partial strips: padded tile rows
    # (padding cells must not count in the strip sums)
    (2, 6, 14, 14, 1024, 1),     # 14x14: two columns of padding per row, two frames per wave
    (2, 11, 14, 14, 1024, 2),    # 5x5 window, ten source frames: three groups of four frames
    (1, 7, 13, 16, 1024, 1),     # 16 wide, odd height: the last strip has one real row
    (2, 6, 9, 24, 1024, 1),      # 24 wide: the second column tile half empty
    (1, 7, 11, 31, 2048, 2),     # 31 wide, 5x5 window
    (2, 6, 12, 12, 1152, 0),     # 1x1 window, 36 K-steps
    (1, 10, 40, 30, 1024, 1),    # 40 strips per frame: the streaming strip reduction ahead of the scores
    # wider than 32: strips of 32 columns with the neighbouring column tiles on both sides
    (1, 6, 9, 48, 1024, 1),      # three column tiles: the second strip of a row is half padding
    (2, 5, 6, 64, 1024, 2),      # whole tiles, 5x5 window
    (1, 7, 5, 100, 2048, 0),     # seven column tiles, 1x1 window
    (1, 6, 7, 45, 1024, 1),      # the emptiest rows the route takes (45 of 64 strip cells)
]


@pytest.mark.parametrize("B,F,H,W,C,r", SHAPES)
def test_confirmed_guess(B, F, H, W, C, r):
    # (a strong contrast between the low-noise frame and the others, so that the guess is clear-cut
    # even with few frames)
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=B, F=F, H=H, W=W, C=C, r=r, max_offset=min(max(r, 1), 2), sigma=1.2,
                                       clean_sigma=0.1)
    batch = make_clip_batch(cfg, seed=4000 + B + F + H + W + C + r)
    _check(batch, cfg, ["confirmed"] * B)


def _with_foreign_guess_channels(cfg, seed):
    """A batch whose clip 0 carries, in the guess channels only, the content of a clip with a different
    low-noise frame: the guess sees that frame as the clear winner, the full rule does not."""
    batch = make_clip_batch(cfg, seed=seed)
    for other_seed in range(seed + 1, seed + 40):
        other = make_clip_batch(cfg.scaled(B=1), seed=other_seed)
        if other.clean_frame[0, 0] != batch.clean_frame[0, 0]:
            idx = guess_channels(cfg.C)
            batch.x[0][..., idx] = other.x[0][..., idx]
            return batch
    raise RuntimeError("no clip with another low-noise frame found")


def test_refuted_guess_is_searched_again():
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=8, C=2048)
    batch = _with_foreign_guess_channels(cfg, seed=4100)
    res = _check(batch, cfg, ["refuted", "confirmed"])
    assert res.anchor_index[0] == batch.clean_frame[0, 0]


def test_refuted_guess_on_a_padded_grid():
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=8, H=14, W=14, C=2048)
    batch = _with_foreign_guess_channels(cfg, seed=4150)
    res = _check(batch, cfg, ["refuted", "confirmed"])
    assert res.anchor_index[0] == batch.clean_frame[0, 0]


def test_unclear_guess_takes_the_two_pass_route():
    # every frame as noisy as the others: no frame stands out, neither to the guess nor to the full rule
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=8, C=1024, clean_sigma=1.0)
    batch = make_clip_batch(cfg, seed=4201)
    _check(batch, cfg, ["fallback", "fallback"])


@pytest.mark.parametrize("H,W", [(16, 16), (9, 24)])
def test_all_three_kinds_in_one_batch(H, W):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=4, F=10, H=H, W=W, C=2048)
    batch = _with_foreign_guess_channels(cfg, seed=4300)
    flat = make_clip_batch(cfg.scaled(clean_sigma=1.0), seed=4300)
    batch.x[2] = flat.x[2]
    batch.amplitude[2], batch.changed[2], batch.offsets[2] = flat.amplitude[2], flat.changed[2], flat.offsets[2]
    _check(batch, cfg, ["refuted", "confirmed", "fallback", "confirmed"])


def test_headline_shape_runs_speculatively_by_default():
    """At the benchmark's size the default setting takes the speculative route (input >= 256 MiB); the
    two settings must agree with the oracle and hence with each other."""
    from oracle import margins
    cfg = CONFIGS["qwen3vl_8b_batched"].scaled(B=4)
    batch = make_clip_batch(cfg)
    res = margins.enforce_margins(batch, cfg.r, cfg.t, want_tokens=False)
    assert all(guess_of(batch.x[b])[1] >= TRUST_GAP and guess_of(batch.x[b])[0] == res.anchor_index[b]
               for b in range(cfg.B))
    for mode in (None, -1):
        _, out = run_gpu(batch.x, cfg.r, cfg.t[0], speculation=mode)
        compare_with_oracle(batch.x, out, res)
