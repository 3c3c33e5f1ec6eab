"""Seeded synthetic workloads standing in for the paper's Brax environments and DAVIS videos.

The paper renders HalfCheetah / Ant / Walker2d / Humanoid states produced by
the Brax simulator and overlays DAVIS-2017 videos (section 2).  Neither is
available offline, so these generators emit articulated-primitive scenes and a
moving-disc video with the same shapes and structure: a kinematic chain, a
quadruped, a humanoid tree, a humanoid plus obstacle with a 3-step frame stack.

This module only prepares INPUTS (scene descriptions as plain dicts, fp32 pose
arrays, uint8 video).  It contains none of the renderer's arithmetic and is the
one module shared by the HIP path's tests/bench and the CPU oracle's tests.
All arrays come from numpy.random.default_rng(250200021 + cfg).
"""
import numpy as np

SEED_BASE = 250200021


def default_scene(width, height, bodies, root_body=0):
    return dict(
        width=width, height=height, bodies=bodies, root_body=root_body,
        fov_y_deg=60.0, cam_offset=(-2.5, 0.0, 1.0), cam_up=(0.0, 0.0, 1.0),
        z_near=0.1, z_far=50.0,
        light_dir=(-0.4, -0.3, 0.85), ambient=0.3, diffuse=0.7,
        ground_enabled=True, ground_cell=1.0, ground_grey=(0.35, 0.65),
        background_rgb=(0.55, 0.70, 0.90),
    )


def capsule(r, h, rgb, n_lon=12, n_lat=6):
    return dict(kind="capsule", shape=(float(r), float(r), float(r), float(h)),
                rgb=tuple(float(c) for c in rgb), n_lon=n_lon, n_lat=n_lat)


def sphere(r, rgb, n_lon=16, n_lat=8):
    return dict(kind="sphere", shape=(float(r), float(r), float(r), 0.0),
                rgb=tuple(float(c) for c in rgb), n_lon=n_lon, n_lat=n_lat)


def box(ex, ey, ez, rgb, n=4):
    return dict(kind="box", shape=(float(ex), float(ey), float(ez), 0.0),
                rgb=tuple(float(c) for c in rgb), n_lon=n, n_lat=0)


def mesh(verts, tris, rgb, scale=(1.0, 1.0, 1.0), mul=None):
    """A caller-supplied triangle mesh body: verts [nv,3] fp32 body-frame positions, tris [nt,3] indices,
    counter-clockwise seen from outside; scale = per-axis factors (the body's shape); mul = per-triangle colour
    multipliers or None."""
    return dict(kind="mesh", shape=(float(scale[0]), float(scale[1]), float(scale[2]), 0.0),
                rgb=tuple(float(c) for c in rgb), n_lon=0, n_lat=0,
                verts=np.ascontiguousarray(verts, dtype=np.float32).reshape(-1, 3),
                tris=np.ascontiguousarray(tris, dtype=np.uint32).reshape(-1, 3),
                mul=None if mul is None else np.ascontiguousarray(mul, dtype=np.float32))


# ------------------------------------------------------------------ procedural meshes (stand-ins for user assets)

def torus_mesh(R=0.3, r=0.1, n_major=16, n_minor=8):
    """Torus around the z axis: (nv, nt) = (n_major*n_minor, 2*n_major*n_minor), outward-facing."""
    u = 2.0 * np.pi * np.arange(n_major) / n_major
    v = 2.0 * np.pi * np.arange(n_minor) / n_minor
    uu, vv = np.meshgrid(u, v, indexing="ij")
    verts = np.stack([(R + r * np.cos(vv)) * np.cos(uu), (R + r * np.cos(vv)) * np.sin(uu), r * np.sin(vv)], axis=-1)
    idx = lambda i, j: (i % n_major) * n_minor + (j % n_minor)
    tris = []
    for i in range(n_major):
        for j in range(n_minor):
            a, b, c, d = idx(i, j), idx(i + 1, j), idx(i + 1, j + 1), idx(i, j + 1)
            tris += [(a, b, c), (a, c, d)]
    return verts.reshape(-1, 3).astype(np.float32), np.array(tris, np.uint32)


def icosphere_mesh(radius=0.2, subdivisions=1):
    """Subdivided icosahedron: 20 * 4^s triangles, vertices pushed to the sphere, outward-facing."""
    t = (1.0 + 5.0 ** 0.5) / 2.0
    v = [(-1, t, 0), (1, t, 0), (-1, -t, 0), (1, -t, 0), (0, -1, t), (0, 1, t), (0, -1, -t), (0, 1, -t),
         (t, 0, -1), (t, 0, 1), (-t, 0, -1), (-t, 0, 1)]
    f = [(0, 11, 5), (0, 5, 1), (0, 1, 7), (0, 7, 10), (0, 10, 11), (1, 5, 9), (5, 11, 4), (11, 10, 2), (10, 7, 6),
         (7, 1, 8), (3, 9, 4), (3, 4, 2), (3, 2, 6), (3, 6, 8), (3, 8, 9), (4, 9, 5), (2, 4, 11), (6, 2, 10), (8, 6, 7),
         (9, 8, 1)]
    v = [np.array(p, np.float64) / np.linalg.norm(p) for p in v]
    for _ in range(subdivisions):
        cache, nf = {}, []

        def mid(a, b):
            key = (min(a, b), max(a, b))
            if key not in cache:
                m = v[a] + v[b]
                v.append(m / np.linalg.norm(m))
                cache[key] = len(v) - 1
            return cache[key]
        for a, b, c in f:
            ab, bc, ca = mid(a, b), mid(b, c), mid(c, a)
            nf += [(a, ab, ca), (b, bc, ab), (c, ca, bc), (ab, bc, ca)]
        f = nf
    return (radius * np.array(v)).astype(np.float32), np.array(f, np.uint32)


def heightfield_mesh(rng, n=12, size=1.0, height=0.15):
    """Open n x n-cell terrain patch in the x-y plane with random heights, facing +z."""
    xs = np.linspace(-size / 2, size / 2, n + 1)
    xx, yy = np.meshgrid(xs, xs, indexing="ij")
    zz = height * rng.uniform(0.0, 1.0, xx.shape)
    verts = np.stack([xx, yy, zz], axis=-1).reshape(-1, 3)
    idx = lambda i, j: i * (n + 1) + j
    tris, mul = [], []
    for i in range(n):
        for j in range(n):
            a, b, c, d = idx(i, j), idx(i + 1, j), idx(i + 1, j + 1), idx(i, j + 1)
            tris += [(a, b, c), (a, c, d)]
            mul += [1.0 if (i + j) & 1 else 0.6] * 2
    return verts.astype(np.float32), np.array(tris, np.uint32), np.array(mul, np.float32)


# ------------------------------------------------------------------ quaternion helpers (w,x,y,z), float64

def q_mul(a, b):
    aw, ax, ay, az = a[..., 0], a[..., 1], a[..., 2], a[..., 3]
    bw, bx, by, bz = b[..., 0], b[..., 1], b[..., 2], b[..., 3]
    return np.stack([aw * bw - ax * bx - ay * by - az * bz,
                     aw * bx + ax * bw + ay * bz - az * by,
                     aw * by - ax * bz + ay * bw + az * bx,
                     aw * bz + ax * by - ay * bx + az * bw], axis=-1)


def q_axis_angle(axis, angle):
    axis = np.asarray(axis, dtype=np.float64)
    angle = np.asarray(angle, dtype=np.float64)
    axis = np.broadcast_to(axis, angle.shape + (3,))
    h = 0.5 * angle
    return np.concatenate([np.cos(h)[..., None], axis * np.sin(h)[..., None]], axis=-1)


def q_rotate(q, v):
    w, x, y, z = q[..., 0], q[..., 1], q[..., 2], q[..., 3]
    vx, vy, vz = v[..., 0], v[..., 1], v[..., 2]
    tx = 2.0 * (y * vz - z * vy)
    ty = 2.0 * (z * vx - x * vz)
    tz = 2.0 * (x * vy - y * vx)
    return np.stack([vx + w * tx + (y * tz - z * ty),
                     vy + w * ty + (z * tx - x * tz),
                     vz + w * tz + (x * ty - y * tx)], axis=-1)


def q_normalize(q):
    return q / np.linalg.norm(q, axis=-1, keepdims=True)


def random_quats(rng, shape):
    return q_normalize(rng.standard_normal(tuple(shape) + (4,)))


def _pose(pos, quat):
    return np.concatenate([pos, q_normalize(quat)], axis=-1).astype(np.float32)


EZ = np.array([0.0, 0.0, 1.0])


# ------------------------------------------------------------------ skeleton descriptions (inputs of the kinematics stage)

def _skeleton(K):
    """All bodies free-floating until hinged: parent -1, slot = index into the free poses / the angles."""
    return dict(parent=np.full(K, -1, np.int32), slot=np.full(K, -1, np.int32), anchor=np.zeros((K, 3), np.float32),
                axis=np.tile(np.array([1.0, 0.0, 0.0], np.float32), (K, 1)), offset=np.zeros((K, 3), np.float32))


def _hinge(skel, k, parent, slot, anchor, axis, offset):
    skel["parent"][k], skel["slot"][k] = parent, slot
    skel["anchor"][k], skel["axis"][k], skel["offset"][k] = anchor, axis, offset


# ------------------------------------------------------------------ the five configurations

def cfg1(B=16):
    """16 envs, 32x32, ground + 4 free-floating capsules (8 longitudes x 4 latitudes per hemisphere)."""
    rng = np.random.default_rng(SEED_BASE + 1)
    K = 4
    r = rng.uniform(0.03, 0.08, K)
    h = rng.uniform(0.1, 0.3, K)
    rgb = rng.uniform(0.2, 0.9, (K, 3))
    bodies = [capsule(r[k], h[k], rgb[k], 8, 4) for k in range(K)]
    pos = np.stack([rng.uniform(-0.5, 0.5, (B, 1, K)), rng.uniform(-0.5, 0.5, (B, 1, K)),
                    rng.uniform(0.2, 0.8, (B, 1, K))], axis=-1)
    quat = random_quats(rng, (B, 1, K))
    return dict(name="cfg1-capsules-32", desc=default_scene(32, 32, bodies), poses=_pose(pos, quat),
                shapes=None, distractor=None, step0=0)


def cfg2(B=256):
    """256 envs, 64x64, planar 7-capsule kinematic chain in the world Y-Z plane."""
    rng = np.random.default_rng(SEED_BASE + 2)
    K = 7
    h = rng.uniform(0.1, 0.25, K)
    rgb = rng.uniform(0.2, 0.9, (K, 3))
    bodies = [capsule(0.046, h[k], rgb[k], 12, 6) for k in range(K)]
    theta = rng.uniform(-0.8, 0.8, (B, K))
    cum = np.cumsum(theta, axis=1)
    pos = np.zeros((B, 1, K, 3))
    quat = np.zeros((B, 1, K, 4))
    start = None
    for i in range(K):
        q = q_axis_angle(np.array([1.0, 0.0, 0.0]), cum[:, i])
        axis = q_rotate(q, np.broadcast_to(EZ, (B, 3)))
        if i == 0:
            centre = np.broadcast_to(np.array([0.0, 0.0, 1.0]), (B, 3)).copy()
        else:
            centre = start + h[i] * axis
        start = centre + h[i] * axis
        pos[:, 0, i] = centre
        quat[:, 0, i] = q
    poses = _pose(pos, quat)
    skel = _skeleton(K)
    skel["slot"][0] = 0  # link 0 is free
    for i in range(1, K):
        _hinge(skel, i, parent=i - 1, slot=i - 1, anchor=(0, 0, h[i - 1]), axis=(1, 0, 0), offset=(0, 0, h[i]))
    fk = dict(skel=skel, free_poses=poses[:, :, :1].copy(), angles=theta[:, None, 1:].astype(np.float32))
    return dict(name="cfg2-chain-64", desc=default_scene(64, 64, bodies), poses=poses,
                shapes=None, distractor=None, step0=0, fk=fk)


def cfg3(B=4096):
    """4096 envs, 64x64, quadruped: sphere torso + 4 two-link legs; colour distractor."""
    rng = np.random.default_rng(SEED_BASE + 3)
    rgb = rng.uniform(0.2, 0.9, (9, 3))
    bodies = [sphere(0.25, rgb[0], 16, 8)] + [capsule(0.05, 0.15, rgb[1 + k], 12, 6) for k in range(8)]
    K = 9
    hl = 0.15
    yaw = rng.uniform(0.0, 2.0 * np.pi, B)
    ang = rng.uniform(-1.0, 1.0, (B, 4, 2))
    q_root = q_axis_angle(EZ, yaw)
    root = np.broadcast_to(np.array([0.0, 0.0, 0.75]), (B, 3))
    pos = np.zeros((B, 1, K, 3))
    quat = np.zeros((B, 1, K, 4))
    pos[:, 0, 0] = root
    quat[:, 0, 0] = q_root
    hips = [(0.18, 0.18, -0.1), (0.18, -0.18, -0.1), (-0.18, 0.18, -0.1), (-0.18, -0.18, -0.1)]
    ey = np.array([0.0, 1.0, 0.0])
    for leg in range(4):
        hip = root + q_rotate(q_root, np.broadcast_to(np.array(hips[leg]), (B, 3)))
        q1 = q_mul(q_root, q_axis_angle(ey, ang[:, leg, 0]))
        d1 = -q_rotate(q1, np.broadcast_to(EZ, (B, 3)))
        q2 = q_mul(q_root, q_axis_angle(ey, ang[:, leg, 0] + ang[:, leg, 1]))
        d2 = -q_rotate(q2, np.broadcast_to(EZ, (B, 3)))
        knee = hip + 2.0 * hl * d1
        pos[:, 0, 1 + 2 * leg] = hip + hl * d1
        quat[:, 0, 1 + 2 * leg] = q1
        pos[:, 0, 2 + 2 * leg] = knee + hl * d2
        quat[:, 0, 2 + 2 * leg] = q2
    dis = dict(mode="color", seed=SEED_BASE + 3, scale=(0.5, 1.5), offset=(-0.2, 0.2))
    poses = _pose(pos, quat)
    skel = _skeleton(K)
    skel["slot"][0] = 0
    for leg in range(4):
        _hinge(skel, 1 + 2 * leg, parent=0, slot=2 * leg, anchor=hips[leg], axis=(0, 1, 0), offset=(0, 0, -hl))
        _hinge(skel, 2 + 2 * leg, parent=1 + 2 * leg, slot=2 * leg + 1, anchor=(0, 0, -hl), axis=(0, 1, 0),
               offset=(0, 0, -hl))
    fk = dict(skel=skel, free_poses=poses[:, :, :1].copy(), angles=ang.reshape(B, 1, 8).astype(np.float32))
    return dict(name="cfg3-quadruped-64", desc=default_scene(64, 64, bodies), poses=poses,
                shapes=None, distractor=dis, step0=0, fk=fk)


def _humanoid_scene(rng):
    """Scene-level humanoid parameters: 13 capsules (torso + 4 limbs x 3 links) + head sphere = 14 bodies."""
    rgb = rng.uniform(0.2, 0.9, (14, 3))
    radii = rng.uniform(0.04, 0.09, (4, 3))
    arm_h = rng.uniform(0.08, 0.14, (2, 3))
    leg_h = rng.uniform(0.12, 0.20, (2, 3))
    half = np.concatenate([arm_h, leg_h], axis=0)  # limb order: L arm, R arm, L leg, R leg
    axes = q_normalize(rng.standard_normal((4, 3, 3)))
    bodies = [capsule(0.09, 0.22, rgb[0], 12, 6), sphere(0.10, rgb[1], 16, 8)]
    for limb in range(4):
        for k in range(3):
            bodies.append(capsule(radii[limb, k], half[limb, k], rgb[2 + limb * 3 + k], 12, 6))
    anchors = np.array([(0.0, 0.22, 0.2), (0.0, -0.22, 0.2), (0.0, 0.1, -0.25), (0.0, -0.1, -0.25)])
    return bodies, half, axes, anchors


def _humanoid_fk(q_root, root, angles, half, axes, anchors):
    """angles [N,4,3] -> positions [N,14,3], quaternions [N,14,4]."""
    N = angles.shape[0]
    pos = np.zeros((N, 14, 3))
    quat = np.zeros((N, 14, 4))
    pos[:, 0] = root
    quat[:, 0] = q_root
    pos[:, 1] = root + q_rotate(q_root, np.broadcast_to(np.array([0.0, 0.0, 0.38]), (N, 3)))
    quat[:, 1] = q_root
    for limb in range(4):
        start = root + q_rotate(q_root, np.broadcast_to(anchors[limb], (N, 3)))
        q = q_root
        for k in range(3):
            q = q_mul(q, q_axis_angle(axes[limb, k], angles[:, limb, k]))
            d = -q_rotate(q, np.broadcast_to(EZ, (N, 3)))
            idx = 2 + limb * 3 + k
            pos[:, idx] = start + half[limb, k] * d
            quat[:, idx] = q
            start = start + 2.0 * half[limb, k] * d
    return pos, quat


def _humanoid_skeleton(K, half, axes, anchors):
    skel = _skeleton(K)
    skel["slot"][0] = 0
    _hinge(skel, 1, parent=0, slot=-1, anchor=(0, 0, 0.38), axis=(1, 0, 0), offset=(0, 0, 0))  # head, rigid
    for limb in range(4):
        for k in range(3):
            idx = 2 + limb * 3 + k
            _hinge(skel, idx, parent=0 if k == 0 else idx - 1, slot=limb * 3 + k,
                   anchor=anchors[limb] if k == 0 else (0, 0, -half[limb, k - 1]), axis=axes[limb, k],
                   offset=(0, 0, -half[limb, k]))
    return skel


def make_video(rng, n_frames, H, W):
    """Synthetic distractor video [n,H,W,3] uint8: dark random-grey background + 6 moving random-colour discs."""
    grey = rng.integers(10, 50, (H, W, 1))
    video = np.broadcast_to(grey, (n_frames, H, W, 3)).astype(np.uint8).copy()
    yy, xx = np.mgrid[0:H, 0:W]
    for _ in range(6):
        rad = rng.uniform(6.0, 18.0)
        colour = rng.integers(0, 256, 3).astype(np.uint8)
        p0 = rng.uniform(0.0, [W, H])
        vel = rng.uniform(-3.0, 3.0, 2)
        for t in range(n_frames):
            cx, cy = (p0 + vel * t) % np.array([W, H])
            dx = np.minimum(np.abs(xx - cx), W - np.abs(xx - cx))
            dy = np.minimum(np.abs(yy - cy), H - np.abs(yy - cy))
            video[t][dx * dx + dy * dy <= rad * rad] = colour
    return video


def cfg4(B=16384):
    """16384 envs, 84x84, humanoid tree (14 bodies); 64-frame video distractor on background and ground."""
    rng = np.random.default_rng(SEED_BASE + 4)
    bodies, half, axes, anchors = _humanoid_scene(rng)
    video = make_video(rng, 64, 84, 84)
    yaw = rng.uniform(0.0, 2.0 * np.pi, B)
    angles = rng.uniform(-1.0, 1.0, (B, 4, 3))
    q_root = q_axis_angle(EZ, yaw)
    root = np.broadcast_to(np.array([0.0, 0.0, 1.25]), (B, 3))
    pos, quat = _humanoid_fk(q_root, root, angles, half, axes, anchors)
    dis = dict(mode="video", seed=SEED_BASE + 4, video=video, alpha=0.5, env_offset=None)
    poses = _pose(pos[:, None], quat[:, None])
    fk = dict(skel=_humanoid_skeleton(14, half, axes, anchors), free_poses=poses[:, :, :1].copy(),
              angles=angles.reshape(B, 1, 12).astype(np.float32))
    return dict(name="cfg4-humanoid-84-video", desc=default_scene(84, 84, bodies),
                poses=poses, shapes=None, distractor=dis, step0=0, fk=fk)


def cfg5(B=65536, S=3):
    """65536 envs x 3 steps, 64x64, humanoid + per-env checker box; colour distractor; frame stack."""
    rng = np.random.default_rng(SEED_BASE + 5)
    bodies, half, axes, anchors = _humanoid_scene(rng)
    box_rgb = rng.uniform(0.2, 0.9, 3)
    bodies = bodies + [box(0.2, 0.2, 0.2, box_rgb, 4)]
    K = 15
    yaw = rng.uniform(0.0, 2.0 * np.pi, B)
    q_root = q_axis_angle(EZ, yaw)
    root = np.broadcast_to(np.array([0.0, 0.0, 1.25]), (B, 3))
    size = rng.uniform(0.2, 0.6, (B, 3))
    ext = 0.5 * size
    box_pos = np.stack([rng.uniform(0.6, 1.6, B), rng.uniform(-0.8, 0.8, B), ext[:, 2]], axis=-1)
    box_q = q_axis_angle(EZ, rng.uniform(0.0, 2.0 * np.pi, B))
    angles = rng.uniform(-1.0, 1.0, (B, 4, 3))
    pos = np.zeros((B, S, K, 3))
    quat = np.zeros((B, S, K, 4))
    all_angles = np.zeros((B, S, 12), np.float32)
    for s in range(S):
        if s > 0:
            angles = angles + rng.normal(0.0, 0.05, (B, 4, 3))
        all_angles[:, s] = angles.reshape(B, 12)
        p, q = _humanoid_fk(q_root, root, angles, half, axes, anchors)
        pos[:, s, :14] = p
        quat[:, s, :14] = q
        pos[:, s, 14] = box_pos
        quat[:, s, 14] = box_q
    shapes = np.zeros((B, K, 4), np.float32)
    for k in range(14):
        shapes[:, k] = np.asarray(bodies[k]["shape"], np.float32)
    shapes[:, 14, :3] = ext.astype(np.float32)
    dis = dict(mode="color", seed=SEED_BASE + 5, scale=(0.5, 1.5), offset=(-0.2, 0.2))
    poses = _pose(pos, quat)
    skel = _humanoid_skeleton(K, half, axes, anchors)
    skel["slot"][14] = 1  # the box is the second free body
    fk = dict(skel=skel, free_poses=np.ascontiguousarray(poses[:, :, [0, 14]]), angles=all_angles)
    return dict(name="cfg5-humanoid-box-64-stack3", desc=default_scene(64, 64, bodies),
                poses=poses, shapes=shapes, distractor=dis, step0=0, fk=fk)


def cfg_mesh(B=64, W=64, H=64):
    """Mesh bodies (the paper's stated next step for its renderer): a free-floating torus, an icosphere and a
    terrain patch given as vertex / index buffers, next to one capsule, with the colour distractor."""
    rng = np.random.default_rng(SEED_BASE + 6)
    tv, tt = torus_mesh(0.3, 0.1, 20, 10)
    iv, it = icosphere_mesh(0.2, 2)
    hv, ht, hm = heightfield_mesh(rng, 12, 1.6, 0.25)
    bodies = [capsule(0.08, 0.25, (0.8, 0.3, 0.3), 12, 6), mesh(tv, tt, (0.3, 0.7, 0.4)),
              mesh(iv, it, (0.4, 0.4, 0.9), scale=(1.0, 1.4, 0.7)), mesh(hv, ht, (0.7, 0.6, 0.4), mul=hm)]
    K = 4
    pos = np.zeros((B, 1, K, 3))
    quat = np.zeros((B, 1, K, 4))
    pos[:, 0, 0] = (0.0, 0.0, 1.0)
    quat[:, 0, 0] = random_quats(rng, (B,))
    for k in (1, 2):
        pos[:, 0, k] = np.array([0.3, 0.0, 1.0]) + rng.uniform(-0.7, 0.7, (B, 3)) * np.array([1.0, 1.0, 0.5])
        quat[:, 0, k] = random_quats(rng, (B,))
    pos[:, 0, 3] = np.array([1.0, 0.0, 0.05]) + rng.uniform(-0.3, 0.3, (B, 3)) * np.array([1.0, 1.0, 0.0])
    quat[:, 0, 3] = q_axis_angle(EZ, rng.uniform(0.0, 2.0 * np.pi, B))
    dis = dict(mode="color", seed=SEED_BASE + 6, scale=(0.5, 1.5), offset=(-0.2, 0.2))
    return dict(name="mesh-bodies-64", desc=default_scene(W, H, bodies), poses=_pose(pos, quat), shapes=None,
                distractor=dis, step0=0)


def _planar_walker(name, seed, B, W, H, torso, legs, torso_pitch):
    """Planar (x-z plane) articulated figure described by its skeleton only: a free torso capsule lying along x
    and `legs` = lists of (radius, half_length) chains hanging from torso anchors, all hinges about y.  Poses
    are not generated here: these workloads enter through the kinematics stage (angles -> poses on the device)."""
    rng = np.random.default_rng(SEED_BASE + seed)
    (tr, th, tz), K = torso, 1 + sum(len(l[1]) for l in legs)
    rgb = rng.uniform(0.2, 0.9, (K, 3))
    bodies = [capsule(tr, th, rgb[0], 12, 6)]
    skel = _skeleton(K)
    skel["slot"][0] = 0
    k, slot = 1, 0
    for anchor_x, links in legs:
        parent, anchor = 0, (0.0, 0.0, anchor_x)  # the torso's own axis is its local z (it is pitched to lie along x)
        for (r, h) in links:
            bodies.append(capsule(r, h, rgb[k], 12, 6))
            _hinge(skel, k, parent=parent, slot=slot, anchor=anchor, axis=(0, 1, 0), offset=(0, 0, -h))
            parent, anchor = k, (0.0, 0.0, -h)
            k += 1
            slot += 1
    free = np.zeros((B, 1, 1, 7), np.float32)
    free[..., :3] = (0.0, 0.0, tz)
    free[:, 0, 0, 3:] = q_axis_angle(np.array([0.0, 1.0, 0.0]), torso_pitch + rng.uniform(-0.2, 0.2, B)).astype(np.float32)
    angles = rng.uniform(-0.9, 0.9, (B, 1, slot))
    first = np.cumsum([0] + [len(l[1]) for l in legs])[:-1]
    angles[:, :, first] -= torso_pitch  # the first link of a leg turns back from the torso's frame: legs hang down
    angles = angles.astype(np.float32)
    desc = default_scene(W, H, bodies)
    desc["cam_offset"] = (0.0, -2.6, 0.6)  # side view, as the planar tasks are usually shown
    return dict(name=name, desc=desc, poses=None, shapes=None, distractor=None, step0=0,
                fk=dict(skel=skel, free_poses=free, angles=angles))


def halfcheetah_like(B=1000, W=64, H=64):
    """Stand-in for the paper's HalfCheetah: torso + back and front leg of three links each (7 bodies, 6 hinges)."""
    leg = [(0.046, 0.145), (0.046, 0.15), (0.046, 0.094)]
    return _planar_walker("halfcheetah-like-64", 7, B, W, H, (0.046, 0.5, 0.7), [(-0.5, leg), (0.5, leg)], np.pi / 2)


def walker2d_like(B=1000, W=64, H=64):
    """Stand-in for the paper's Walker2d: upright torso + two legs of thigh, shin, foot (7 bodies, 6 hinges)."""
    leg = [(0.05, 0.225), (0.04, 0.25), (0.06, 0.1)]
    return _planar_walker("walker2d-like-64", 8, B, W, H, (0.05, 0.2, 1.25), [(-0.2, leg), (-0.2, leg)], 0.0)


def ant_like(B=1000):
    """Stand-in for the paper's Ant: the quadruped of configuration 3 without its distractor."""
    w = cfg3(B)
    return dict(w, name="ant-like-64", distractor=None)


def humanoid_like(B=1000):
    """Stand-in for the paper's Humanoid: the 14-body tree of configuration 4 at 64x64 without its distractor."""
    w = cfg4(B)
    desc = dict(w["desc"], width=64, height=64)
    return dict(w, name="humanoid-like-64", desc=desc, distractor=None)


PAPER_ENVIRONMENTS = {"halfcheetah": halfcheetah_like, "ant": ant_like, "walker2d": walker2d_like, "humanoid": humanoid_like}

CONFIGS = {1: cfg1, 2: cfg2, 3: cfg3, 4: cfg4, 5: cfg5}


def make(cfg, B=None):
    """Workload `cfg` in 1..5, optionally at a reduced (or enlarged) environment count."""
    fn = CONFIGS[int(cfg)]
    return fn() if B is None else fn(B)


def random_scene(seed, B=4):
    """A seeded random scene for parity fuzzing: image shape (packed and unpacked store paths, banded or not),
    camera (offset, field of view, with or without roll), ground, a mix of capsules / spheres / boxes of random
    size and tessellation at random distances (so that triangles of every raster bin occur), free random poses,
    optional per-environment shapes and any of the three distractor modes."""
    rng = np.random.default_rng(SEED_BASE + 1000 + int(seed))
    W = int(rng.choice([24, 33, 40, 64, 84, 96, 110]))
    H = int(rng.choice([16, 31, 48, 64, 84, 100]))
    K = int(rng.integers(1, 9))
    bodies = []
    for _ in range(K):
        rgb = rng.uniform(0.1, 1.0, 3)
        kind = int(rng.integers(0, 3))
        if kind == 0:
            bodies.append(capsule(rng.uniform(0.03, 0.3), rng.uniform(0.0, 0.5), rgb, int(rng.integers(3, 14)), int(rng.integers(1, 7))))
        elif kind == 1:
            bodies.append(sphere(rng.uniform(0.05, 0.6), rgb, int(rng.integers(3, 18)), int(rng.integers(1, 9))))
        else:
            e = rng.uniform(0.05, 0.6, 3)
            bodies.append(box(e[0], e[1], e[2], rgb, int(rng.integers(1, 6))))
    desc = default_scene(W, H, bodies, root_body=int(rng.integers(0, K)))
    off = rng.uniform(-1.0, 1.0, 3)
    off = off / np.linalg.norm(off) * rng.uniform(0.8, 4.0)
    off[2] = abs(off[2]) * 0.7 + 0.1
    desc.update(fov_y_deg=float(rng.uniform(25.0, 95.0)), cam_offset=tuple(float(x) for x in off),
                ground_enabled=bool(rng.random() < 0.8), ground_cell=float(rng.choice([1.0, 1.0, 0.37, 2.5])),
                z_far=float(rng.choice([50.0, 6.0])), light_dir=tuple(float(x) for x in rng.uniform(-1.0, 1.0, 3) + np.array([0, 0, 0.2])))
    if rng.random() < 0.4:  # camera roll
        desc["cam_up"] = (float(rng.uniform(-0.4, 0.4)), float(rng.uniform(-0.4, 0.4)), 1.0)
    S = int(rng.integers(1, 4))
    poses = np.zeros((B, S, K, 7), np.float32)
    poses[..., :3] = rng.uniform([-0.8, -0.8, 0.1], [0.8, 0.8, 1.6], (B, S, K, 3))
    q = rng.standard_normal((B, S, K, 4))
    poses[..., 3:] = q / np.linalg.norm(q, axis=-1, keepdims=True)
    shapes = None
    if rng.random() < 0.5:
        base = np.array([b["shape"] for b in bodies], np.float32)
        shapes = (base[None] * rng.uniform(0.6, 1.5, (B, K, 1))).astype(np.float32)
    mode = int(rng.integers(0, 3))
    dis = None
    if mode == 1:
        lo, span = float(rng.uniform(0.3, 1.0)), float(rng.uniform(0.0, 1.0))
        olo, ospan = float(rng.uniform(-0.4, 0.1)), float(rng.uniform(0.0, 0.5))
        dis = dict(mode="color", seed=int(rng.integers(0, 2**62)), scale=(lo, lo + span), offset=(olo, olo + ospan))
    elif mode == 2:
        n = int(rng.integers(1, 6))
        dis = dict(mode="video", seed=int(rng.integers(0, 2**62)), alpha=float(rng.choice([0.5, 0.25, 1.0])),
                   video=rng.integers(0, 256, (n, H, W, 3), dtype=np.uint8))
    return dict(name=f"random-{seed}", desc=desc, poses=poses, shapes=shapes, distractor=dis)
