"""Pins for the oracle's counter-based generator, its two distractors and whole-path invariants.

The paper (section 2) fixes: colour distractor = the whole frame's colour bias
changes at every step; video distractor = step t+1 shows video frame t+1;
everything reproducible from a seed.
"""
import numpy as np
import pytest

from paper_2502_00021_amd import workloads as wl

BG = 0xFFFFFFFF
GROUND = 0xFFFFFFFE
M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def _encrypt(seed, ctr):
    """The 10-round 4x32 multiply/xor network with Python big integers."""
    k0, k1 = seed & MASK, (seed >> 32) & MASK
    c0, c1, c2, c3 = ctr
    for r in range(10):
        if r:
            k0, k1 = (k0 + W0) & MASK, (k1 + W1) & MASK
        p0, p1 = M0 * c0, M1 * c2
        c0, c1, c2, c3 = (p1 >> 32) ^ c1 ^ k0, p1 & MASK, (p0 >> 32) ^ c3 ^ k1, p0 & MASK
    return c0, c1, c2, c3


def _decrypt(seed, out):
    """Inverse network: each round is a bijection because the multipliers are odd (invertible mod 2^32)."""
    i0, i1 = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    keys = [((seed & MASK) + r * W0) & MASK for r in range(10)], [(((seed >> 32) & MASK) + r * W1) & MASK for r in range(10)]
    n0, n1, n2, n3 = out
    for r in reversed(range(10)):
        c0 = (n3 * i0) & MASK
        c2 = (n1 * i1) & MASK
        c1 = n0 ^ ((M1 * c2) >> 32) ^ keys[0][r]
        c3 = n2 ^ ((M0 * c0) >> 32) ^ keys[1][r]
        n0, n1, n2, n3 = c0, c1, c2, c3
    return n0, n1, n2, n3


def test_generator_matches_the_published_known_answers(orc):
    """The 10-round 4x32 multiply/xor network IS Philox-4x32-10: the published known-answer vectors come out."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        c = [int(x, 16) for x in r[:4]]
        key = int(r[4], 16) | (int(r[5], 16) << 32)
        assert [int(x) for x in orc.philox(key, *c)] == [int(x, 16) for x in r[6:]]


def test_generator_is_the_described_bijection(orc):
    rng = np.random.default_rng(1)
    for _ in range(300):
        seed = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        ctr = tuple(int(v) for v in rng.integers(0, 1 << 32, 4))
        got = tuple(int(v) for v in orc.philox(seed, *ctr))
        assert got == _encrypt(seed, ctr)
        assert _decrypt(seed, got) == ctr  # invertible => no two counters collide under one key
    # edge words
    for ctr in [(0, 0, 0, 0), (MASK, MASK, MASK, MASK), (1, 0, 0, 0), (0, 0, 1, 0)]:
        for seed in (0, (1 << 64) - 1, 250200024):
            assert tuple(int(v) for v in orc.philox(seed, *ctr)) == _encrypt(seed, ctr)


def test_generator_statistics_and_sensitivity(orc):
    n = 1 << 16
    words = np.array([orc.philox(12345, e, s, 0, 0) for e in range(256) for s in range(n // 256)], dtype=np.uint64)
    flat = words.reshape(-1)
    assert len(np.unique(words.view([("", words.dtype)] * 4))) == n  # distinct counters -> distinct blocks
    u = (flat >> np.uint64(8)).astype(np.float64) / (1 << 24)
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / len(u))
    assert abs(u.var() - 1 / 12) < 1e-3
    hist = np.bincount((u * 64).astype(int), minlength=64)
    chi2 = ((hist - len(u) / 64) ** 2 / (len(u) / 64)).sum()
    assert chi2 < 120  # 63 dof: p(>120) ~ 2e-5
    bits = ((flat[:, None] >> np.arange(32, dtype=np.uint64)[None, :]) & np.uint64(1)).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 0.01)
    # avalanche: flipping one counter/key bit flips about half of the 128 output bits
    base = orc.philox(99, 5, 7, 0, 0)
    for other in (orc.philox(99, 4, 7, 0, 0), orc.philox(99, 5, 6, 0, 0), orc.philox(99, 5, 7, 1, 0), orc.philox(98, 5, 7, 0, 0),
                  orc.philox(99 + (1 << 32), 5, 7, 0, 0)):
        flipped = sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(base, other))
        assert 35 < flipped < 93
    assert np.array_equal(base, orc.philox(99, 5, 7, 0, 0))


def test_u01(orc):
    assert orc.u01(0) == 0.0
    assert orc.u01(0xFF) == 0.0
    assert orc.u01(0x100) == 2.0 ** -24
    assert orc.u01(MASK) == 1.0 - 2.0 ** -24
    assert orc.u01(0x80000000) == 0.5


# ---------------------------------------------------------------- distractors on a small scene

@pytest.fixture(scope="module")
def small():
    w = wl.make(3, B=6)
    w["desc"]["width"] = w["desc"]["height"] = 40
    return w


def _u8(c):
    return np.floor(np.float32(c) * np.float32(255.0) + np.float32(0.5)).astype(np.uint8)


def test_colour_identity_and_per_step_change(orc, small):
    s = orc.Scene(small["desc"])
    plain = s.render(small["poses"])
    ident = s.render(small["poses"], distractor=dict(mode="color", seed=3, scale=(1.0, 1.0), offset=(0.0, 0.0)))
    assert np.array_equal(plain["frames"], ident["frames"]) and np.array_equal(plain["ids"], ident["ids"])
    d = dict(mode="color", seed=3, scale=(0.5, 1.5), offset=(-0.2, 0.2))
    a = s.render(small["poses"], distractor=d, step0=10)
    b = s.render(small["poses"], distractor=d, step0=11)
    assert np.array_equal(a["ids"], plain["ids"])  # geometry untouched
    for e in range(6):
        assert not np.array_equal(a["frames"][e], b["frames"][e])      # new draw each step
    # every env gets its own draw: background bytes differ between envs
    bgpix = [tuple(a["frames"][e, 0][plain["ids"][e, 0] == BG][0]) for e in range(6)]
    assert len(set(bgpix)) == 6
    # same (seed, env, step) => same bytes; different seed => different
    assert np.array_equal(a["frames"], s.render(small["poses"], distractor=d, step0=10)["frames"])
    assert not np.array_equal(a["frames"], s.render(small["poses"], distractor=dict(d, seed=4), step0=10)["frames"])


def test_misspelt_distractor_fields_are_rejected(orc, small):
    """A key that neither wrapper knows would silently leave its default (no jitter) in place on both sides."""
    import pytest
    from paper_2502_00021_amd import pxr, workloads as wl
    s = orc.Scene(small["desc"])
    with pytest.raises(KeyError):
        s.render(small["poses"], distractor=dict(mode="color", seed=3, scale_lo=0.5, scale_hi=1.5))
    sc = pxr.Scene.__new__(pxr.Scene)  # (no device here: the keys are checked before the library is called)
    with pytest.raises(ValueError):
        pxr.Scene.apply_distractor(sc, dict(mode="color", seed=3, scale_lo=0.5))
    # the fuzz generator's colour scenes really jitter
    seen = 0
    for seed in range(40):
        d = wl.random_scene(seed)["distractor"]
        if d and d["mode"] == "color":
            assert d["scale"][1] >= d["scale"][0] > 0.0 and d["offset"][1] >= d["offset"][0]
            seen += 1
    assert seen >= 5


def test_colour_distractor_values_from_the_generator(orc, small):
    """Background pixels carry exactly clamp(bg*scale+offset) with scale/offset drawn from streams 0 and 1."""
    s = orc.Scene(small["desc"])
    seed, step = 77, 5
    d = dict(mode="color", seed=seed, scale=(0.5, 1.5), offset=(-0.2, 0.2))
    out = s.render(small["poses"], distractor=d, step0=step, env0=100)
    bg = np.array(small["desc"]["background_rgb"], np.float32)
    for e in range(6):
        r0, r1 = orc.philox(seed, 100 + e, step, 0, 0), orc.philox(seed, 100 + e, step, 1, 0)
        scale = np.array([np.float32(0.5) + np.float32(orc.u01(r0[c])) * np.float32(1.0) for c in range(3)])
        offs = np.array([np.float32(orc.u01(r1[c])) * np.float32(0.4) + np.float32(-0.2) for c in range(3)])
        assert np.all((scale >= 0.5) & (scale < 1.5)) and np.all((offs >= -0.2) & (offs < 0.2))
        expect = 255.0 * np.clip(bg.astype(np.float64) * scale + offs, 0.0, 1.0)
        px = out["frames"][e, 0][out["ids"][e, 0] == BG]
        assert np.all(px == px[0])
        assert np.all(np.abs(px[0].astype(np.float64) - expect) <= 0.5 + 1e-3)


def test_colour_clamp_at_extremes(orc, small):
    s = orc.Scene(small["desc"])
    hi = s.render(small["poses"], distractor=dict(mode="color", seed=1, scale=(50.0, 50.0), offset=(1.0, 1.0)))
    lo = s.render(small["poses"], distractor=dict(mode="color", seed=1, scale=(1.0, 1.0), offset=(-5.0, -5.0)))
    assert np.all(hi["frames"] == 255) and np.all(lo["frames"] == 0)


def test_video_alpha_limits_mask_and_frame_advance(orc, small):
    s = orc.Scene(small["desc"])
    H = W = 40
    rng = np.random.default_rng(8)
    video = rng.integers(0, 256, (5, H, W, 3), dtype=np.uint8)
    eo = np.array([0, 1, 2, 3, 4, 7], np.uint32)
    plain = s.render(small["poses"])
    masked = (plain["ids"] == BG) | (plain["ids"] == GROUND)
    assert masked.any() and (~masked).any()
    a0 = s.render(small["poses"], distractor=dict(mode="video", video=video, alpha=0.0, env_offset=eo))
    assert np.array_equal(a0["frames"], plain["frames"])
    for step in (0, 1, 4, 13):
        a1 = s.render(small["poses"], distractor=dict(mode="video", video=video, alpha=1.0, env_offset=eo), step0=step)
        for e in range(6):
            fi = (int(eo[e]) + step) % 5  # frame index advances by one per step, wraps
            m = masked[e, 0]
            assert np.array_equal(a1["frames"][e, 0][m], video[fi][m])
            assert np.array_equal(a1["frames"][e, 0][~m], plain["frames"][e, 0][~m])
    half = s.render(small["poses"], distractor=dict(mode="video", video=video, alpha=0.5, env_offset=eo), step0=2)
    for e in range(6):
        m = masked[e, 0]
        fi = (int(eo[e]) + 2) % 5
        mix = 0.5 * (plain["frames"][e, 0][m].astype(np.float64) + video[fi][m].astype(np.float64))
        assert np.all(np.abs(half["frames"][e, 0][m].astype(np.float64) - mix) <= 1.0)
    # offsets drawn from the generator when none are given: stream 2, step word 0xFFFFFFFF, modulo n_frames
    auto = s.render(small["poses"], distractor=dict(mode="video", video=video, alpha=1.0, seed=55), step0=3, env0=9)
    for e in range(6):
        fi = (int(orc.philox(55, 9 + e, MASK, 2, 0)[0]) % 5 + 3) % 5
        m = masked[e, 0]
        assert np.array_equal(auto["frames"][e, 0][m], video[fi][m])


def test_video_sets_play_one_clip_per_environment(orc, small):
    """Several clips: environment e shows clip c(e) (given, reduced modulo the count, or drawn from stream 3 at
    step word 0xFFFFFFFF), i.e. exactly what a single-clip render with that clip shows."""
    s = orc.Scene(small["desc"])
    H = W = 40
    rng = np.random.default_rng(9)
    clips = rng.integers(0, 256, (4, 5, H, W, 3), dtype=np.uint8)
    eo = np.array([0, 1, 2, 3, 4, 7], np.uint32)
    ev = np.array([3, 0, 1, 2, 6, 9], np.uint32)  # 6 -> 2, 9 -> 1
    got = s.render(small["poses"], distractor=dict(mode="video", video=clips, alpha=0.6, env_offset=eo, env_video=ev), step0=4)
    for e in range(6):
        one = s.render(small["poses"][e:e + 1], env0=e, step0=4,
                       distractor=dict(mode="video", video=clips[int(ev[e]) % 4], alpha=0.6, env_offset=eo[e:e + 1]))
        assert np.array_equal(got["frames"][e], one["frames"][0])
    auto = s.render(small["poses"], distractor=dict(mode="video", video=clips, alpha=1.0, seed=55), step0=3, env0=9)
    plain = s.render(small["poses"])
    masked = (plain["ids"] == BG) | (plain["ids"] == GROUND)
    for e in range(6):
        clip = int(orc.philox(55, 9 + e, MASK, 3, 0)[0]) % 4
        fi = (int(orc.philox(55, 9 + e, MASK, 2, 0)[0]) % 5 + 3) % 5
        m = masked[e, 0]
        assert np.array_equal(auto["frames"][e, 0][m], clips[clip, fi][m])
    # the drawn clip index is spread over the set
    picks = [int(orc.philox(1, e, MASK, 3, 0)[0]) % 4 for e in range(4000)]
    assert min(np.bincount(picks, minlength=4)) > 900
    # one clip given as a set of one
    a = s.render(small["poses"], distractor=dict(mode="video", video=clips[:1], alpha=0.5, seed=2), step0=1)
    b = s.render(small["poses"], distractor=dict(mode="video", video=clips[0], alpha=0.5, seed=2), step0=1)
    assert np.array_equal(a["frames"], b["frames"])


# ---------------------------------------------------------------- whole path

@pytest.mark.parametrize("cfg,B", [(1, 16), (2, 6), (3, 6), (4, 4), (5, 4)])
def test_determinism_split_and_slice_invariance(orc, cfg, B):
    w = wl.make(cfg, B=B)
    s = orc.Scene(w["desc"])
    full = s.render(w["poses"], w["shapes"], distractor=w["distractor"], step0=4)
    again = s.render(w["poses"], w["shapes"], distractor=w["distractor"], step0=4)
    assert np.array_equal(full["frames"], again["frames"]) and np.array_equal(full["ids"], again["ids"])
    # env e rendered alone (with its global index) equals its slice of the batch
    e = B // 2
    sh = None if w["shapes"] is None else w["shapes"][e:e + 1]
    one = s.render(w["poses"][e:e + 1], sh, distractor=w["distractor"], step0=4, env0=e)
    assert np.array_equal(one["frames"][0], full["frames"][e]) and np.array_equal(one["ids"][0], full["ids"][e])
    # steps rendered in two calls equal one call (resume = pass the same step0)
    S = w["poses"].shape[1]
    if S > 1:
        first = s.render(w["poses"][:, :1], w["shapes"], distractor=w["distractor"], step0=4)
        rest = s.render(w["poses"][:, 1:], w["shapes"], distractor=w["distractor"], step0=5)
        assert np.array_equal(np.concatenate([first["frames"], rest["frames"]], axis=1), full["frames"])
    # triangle submission order is irrelevant
    rng = np.random.default_rng(cfg)
    perm = s.render(w["poses"], w["shapes"], distractor=w["distractor"], step0=4, order=rng.permutation(s.T))
    assert np.array_equal(perm["frames"], full["frames"]) and np.array_equal(perm["ids"], full["ids"])


def test_config_sizes_match_the_closed_forms(orc):
    expect = {1: (264, 512), 2: (1022, 2016), 3: (1410, 2784), 4: (2140, 4224), 5: (2290, 4416)}
    for cfg, (V, T) in expect.items():
        s = orc.Scene(wl.make(cfg, B=1)["desc"])
        assert (s.V, s.T) == (V, T)
