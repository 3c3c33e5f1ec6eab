"""ctypes loader for the CPU oracle (test infrastructure, never the product path).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg import
this module.  It compiles oracle/orc.cpp with g++ on first use and exposes thin
numpy wrappers around the C functions declared in oracle/orc.h.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "orc.cpp")
_LIB = os.path.join(_HERE, "liborc.so")

ID_GROUND = 0xFFFFFFFE
ID_BG = 0xFFFFFFFF
KINDS = {"capsule": 0, "sphere": 1, "box": 2, "mesh": 3}
MODES = {"none": 0, "color": 1, "video": 2}

CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force=False, extra_flags=(), out=None):
    out = out or _LIB
    if (not force and os.path.exists(out)
            and os.path.getmtime(out) >= max(os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "orc.h")))):
        return out
    subprocess.check_call(["g++", *CXXFLAGS, *extra_flags, "-o", out, _SRC])
    return out


class _Distractor(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("seed", C.c_uint64),
                ("scale_lo", C.c_float), ("scale_hi", C.c_float),
                ("offset_lo", C.c_float), ("offset_hi", C.c_float),
                ("video", C.c_void_p), ("n_frames", C.c_uint32), ("alpha", C.c_float),
                ("env_offset", C.c_void_p), ("n_videos", C.c_uint32), ("env_video", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        vp, u32, u64, f32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_float
        _lib.orc_scene_create.restype = vp
        _lib.orc_scene_create.argtypes = [u32, u32, u32, u32] + [vp] * 9
        _lib.orc_scene_create_meshes.restype = vp
        _lib.orc_scene_create_meshes.argtypes = [u32, u32, u32, u32] + [vp] * 14
        _lib.orc_scene_destroy.argtypes = [vp]
        _lib.orc_scene_destroy.restype = None
        _lib.orc_scene_counts.argtypes = [vp, vp, vp]
        _lib.orc_scene_counts.restype = None
        _lib.orc_scene_mesh.argtypes = [vp] * 7
        _lib.orc_scene_mesh.restype = None
        _lib.orc_scene_camera.argtypes = [vp] * 7
        _lib.orc_scene_camera.restype = None
        _lib.orc_vertex_stage.argtypes = [vp] * 8
        _lib.orc_vertex_stage.restype = None
        _lib.orc_raster.argtypes = [u32, u32, u32, vp, vp, vp, vp, u32, vp, vp, u32, vp, vp, vp]
        _lib.orc_raster.restype = None
        _lib.orc_render.argtypes = [vp, vp, vp, u32, u32, u32, u32, vp, vp, vp, vp, vp]
        _lib.orc_render.restype = C.c_int
        _lib.orc_philox.argtypes = [u64, u32, u32, u32, u32, vp]
        _lib.orc_philox.restype = None
        _lib.orc_u01.argtypes = [u32]
        _lib.orc_u01.restype = f32
        _lib.orc_fk.argtypes = [u32] + [vp] * 8
        _lib.orc_fk.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


class Scene:
    """Oracle scene built from the plain-dict scene description used by the workload generators."""

    def __init__(self, desc):
        L = lib()
        bodies = desc["bodies"]
        K = len(bodies)
        kinds = np.array([KINDS[b["kind"]] for b in bodies], dtype=np.uint32)
        shapes = _f32([b["shape"] for b in bodies]).reshape(K, 4)
        rgbs = _f32([b["rgb"] for b in bodies]).reshape(K, 3)
        nlon = np.array([b["n_lon"] for b in bodies], dtype=np.uint32)
        nlat = np.array([b.get("n_lat", 0) for b in bodies], dtype=np.uint32)
        cam = _f32([desc["fov_y_deg"], *desc["cam_offset"], *desc["cam_up"], desc["z_near"], desc["z_far"]])
        light = _f32([*desc["light_dir"], desc["ambient"], desc["diffuse"]])
        ground = _f32([1.0 if desc["ground_enabled"] else 0.0, desc["ground_cell"], *desc["ground_grey"]])
        bg = _f32(desc["background_rgb"])
        self.W, self.H, self.K = int(desc["width"]), int(desc["height"]), K
        meshes = [b for b in bodies if b["kind"] == "mesh"]
        mesh_nv = np.array([len(b["verts"]) if b["kind"] == "mesh" else 0 for b in bodies], dtype=np.uint32)
        mesh_nt = np.array([len(b["tris"]) if b["kind"] == "mesh" else 0 for b in bodies], dtype=np.uint32)
        if meshes:
            mv = _f32(np.concatenate([np.asarray(b["verts"], np.float32).reshape(-1, 3) for b in meshes]))
            mt = np.ascontiguousarray(np.concatenate([np.asarray(b["tris"]).reshape(-1, 3) for b in meshes]), dtype=np.uint32)
            mm = _f32(np.concatenate([np.ones(len(b["tris"]), np.float32) if b.get("mul") is None
                                      else np.asarray(b["mul"], np.float32) for b in meshes]))
        else:
            mv = mt = mm = None
        self._h = L.orc_scene_create_meshes(self.W, self.H, K, int(desc["root_body"]), _p(kinds), _p(shapes), _p(rgbs),
                                            _p(nlon), _p(nlat), _p(cam), _p(light), _p(ground), _p(bg),
                                            _p(mesh_nv), _p(mesh_nt), _p(mv), _p(mt), _p(mm))
        if not self._h:
            raise ValueError("orc_scene_create rejected the scene description")
        nv, nt = C.c_uint32(), C.c_uint32()
        L.orc_scene_counts(self._h, C.byref(nv), C.byref(nt))
        self.V, self.T = nv.value, nt.value

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_scene_destroy(self._h)
            self._h = None

    def mesh(self):
        uv = np.empty((self.V, 4), np.float32)
        tris = np.empty((self.T, 3), np.uint32)
        nrm = np.empty((self.T, 3), np.float32)
        mul = np.empty(self.T, np.float32)
        tb = np.empty(self.T, np.uint32)
        vb = np.empty(self.V, np.uint32)
        lib().orc_scene_mesh(self._h, _p(uv), _p(tris), _p(nrm), _p(mul), _p(tb), _p(vb))
        return dict(uverts=uv, tris=tris, normals=nrm, mul=mul, tri_body=tb, vert_body=vb)

    def camera(self):
        Rv = np.empty((3, 3), np.float32)
        f = np.empty(1, np.float32)
        cx = np.empty(self.W, np.float32)
        cy = np.empty(self.H, np.float32)
        gs = np.empty(2, np.float32)
        l = np.empty(3, np.float32)
        lib().orc_scene_camera(self._h, _p(Rv), _p(f), _p(cx), _p(cy), _p(gs), _p(l))
        return dict(Rv=Rv, f=float(f[0]), cx=cx, cy=cy, gs=gs, l=l)

    def vertex_stage(self, poses, shapes=None):
        poses = _f32(poses).reshape(self.K, 7)
        shapes = None if shapes is None else _f32(shapes).reshape(self.K, 4)
        X = np.empty(self.V, np.int32)
        Y = np.empty(self.V, np.int32)
        D = np.empty(self.V, np.float32)
        rej = np.empty(self.V, np.uint8)
        eye = np.empty(3, np.float32)
        lib().orc_vertex_stage(self._h, _p(poses), _p(shapes), _p(X), _p(Y), _p(D), _p(rej), _p(eye))
        return dict(X=X, Y=Y, D=D, rejected=rej, eye=eye)

    def render(self, poses, shapes=None, step0=0, env0=0, distractor=None, order=None,
               want_ids=True, want_depth=False):
        poses = _f32(poses)
        B, S = poses.shape[0], poses.shape[1]
        assert poses.shape == (B, S, self.K, 7), poses.shape
        if shapes is not None:
            shapes = _f32(shapes)
            assert shapes.shape == (B, self.K, 4)
        frames = np.empty((B, S, self.H, self.W, 3), np.uint8)
        ids = np.empty((B, S, self.H, self.W), np.uint32) if want_ids else None
        dep = np.empty((B, S, self.H, self.W), np.uint32) if want_depth else None
        dis, keep = _make_distractor(distractor, B)
        if order is not None:
            order = np.ascontiguousarray(order, dtype=np.uint32)
            assert order.shape == (self.T,)
        rc = lib().orc_render(self._h, _p(poses), _p(shapes), B, S, int(step0), int(env0),
                              C.byref(dis) if dis is not None else None, _p(order), _p(frames), _p(ids), _p(dep))
        del keep
        if rc != 0:
            raise ValueError("orc_render rejected its arguments")
        out = dict(frames=frames)
        if want_ids:
            out["ids"] = ids
        if want_depth:
            out["depth_bits"] = dep
        return out


def _make_distractor(d, B):
    if d is None or d.get("mode", "none") == "none":
        return None, None
    for key in d:
        if key not in ("mode", "seed", "scale", "offset", "video", "alpha", "env_offset", "env_video"):
            raise KeyError(f"distractor description has no field {key!r}")
    s = _Distractor()
    s.mode = MODES[d["mode"]]
    s.seed = int(d.get("seed", 0))
    s.scale_lo, s.scale_hi = d.get("scale", (1.0, 1.0))
    s.offset_lo, s.offset_hi = d.get("offset", (0.0, 0.0))
    keep = []
    if d["mode"] == "video":
        v = np.ascontiguousarray(d["video"], dtype=np.uint8)
        keep.append(v)
        s.video = v.ctypes.data
        if v.ndim == 5:  # several clips [n_videos, n_frames, H, W, 3]
            s.n_videos, s.n_frames = v.shape[0], v.shape[1]
            ev = d.get("env_video")
            if ev is not None:
                ev = np.ascontiguousarray(ev, dtype=np.uint32)
                assert ev.shape == (B,)
                keep.append(ev)
                s.env_video = ev.ctypes.data
        else:
            s.n_frames = v.shape[0]
        s.alpha = float(d.get("alpha", 0.5))
        eo = d.get("env_offset")
        if eo is not None:
            eo = np.ascontiguousarray(eo, dtype=np.uint32)
            assert eo.shape == (B,)
            keep.append(eo)
            s.env_offset = eo.ctypes.data
    return s, keep


def raster(W, H, X, Y, D, tris, rejected=None, order=None, cull=0):
    """Raster an arbitrary snapped triangle soup; returns ids, depth_bits, cover (each [H,W])."""
    X = np.ascontiguousarray(X, dtype=np.int32)
    Y = np.ascontiguousarray(Y, dtype=np.int32)
    D = _f32(D)
    tris = np.ascontiguousarray(tris, dtype=np.uint32).reshape(-1, 3)
    nv, nt = X.shape[0], tris.shape[0]
    rej = np.zeros(nv, np.uint8) if rejected is None else np.ascontiguousarray(rejected, dtype=np.uint8)
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.uint32)
    ids = np.empty((H, W), np.uint32)
    dep = np.empty((H, W), np.uint32)
    cov = np.empty((H, W), np.uint32)
    lib().orc_raster(W, H, nv, _p(X), _p(Y), _p(D), _p(rej), nt, _p(tris), _p(order), int(cull),
                     _p(ids), _p(dep), _p(cov))
    return ids, dep, cov


def philox(seed, c0, c1, c2, c3):
    out = np.empty(4, np.uint32)
    lib().orc_philox(int(seed), int(c0), int(c1), int(c2), int(c3), _p(out))
    return out


def u01(x):
    return float(lib().orc_u01(int(x)))


def fk(skel, free_poses, angles):
    """Forward kinematics over a batch: skel = dict(parent, slot, anchor, axis, offset) of length-K arrays,
    free_poses [..., F, 7], angles [..., J] -> poses [..., K, 7] (fp32)."""
    parent = np.ascontiguousarray(skel["parent"], dtype=np.int32)
    slot = np.ascontiguousarray(skel["slot"], dtype=np.int32)
    anchor, axis, offset = _f32(skel["anchor"]), _f32(skel["axis"]), _f32(skel["offset"])
    K = parent.shape[0]
    free_poses, angles = _f32(free_poses), _f32(angles)
    lead = free_poses.shape[:-2]
    fp = free_poses.reshape(-1, free_poses.shape[-2], 7)
    an = angles.reshape(fp.shape[0], -1)
    out = np.empty((fp.shape[0], K, 7), np.float32)
    for n in range(fp.shape[0]):
        rc = lib().orc_fk(K, _p(parent), _p(slot), _p(anchor), _p(axis), _p(offset), _p(fp[n]), _p(an[n]), _p(out[n]))
        if rc:
            raise ValueError("orc_fk rejected the skeleton")
    return out.reshape(*lead, K, 7)
