"""ctypes binding of libpxr.so — argument marshalling only; every step runs in the HIP library.

Mirrors include/pxr.h one to one: create_scene / destroy_scene /
apply_distractor / render_batch, set_skeleton / pose_batch /
render_batch_kinematic (+ scene_info, set_block_threads, host_tables).  PyTorch is used only to hold device memory and name the stream.
There is no fallback: a missing library or a failing call raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpxr.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_OOM, ERR_DEVICE = range(5)
ID_GROUND = 0xFFFFFFFE
ID_BG = 0xFFFFFFFF
KINDS = {"capsule": 0, "sphere": 1, "box": 2, "mesh": 3}
MODES = {"none": 0, "color": 1, "video": 2}


class PxrError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"pxr error {code}: {message}")
        self.code = code


class BodyDesc(C.Structure):
    _fields_ = [("type", C.c_uint32), ("shape", C.c_float * 4), ("rgb", C.c_float * 3),
                ("n_lon", C.c_uint32), ("n_lat", C.c_uint32),
                ("mesh_verts", C.c_void_p), ("mesh_tris", C.c_void_p), ("mesh_tri_mul", C.c_void_p),
                ("n_mesh_verts", C.c_uint32), ("n_mesh_tris", C.c_uint32)]


class SceneDesc(C.Structure):
    _fields_ = [("width", C.c_uint32), ("height", C.c_uint32), ("n_bodies", C.c_uint32), ("root_body", C.c_uint32),
                ("bodies", C.POINTER(BodyDesc)),
                ("fov_y_deg", C.c_float), ("cam_offset", C.c_float * 3), ("cam_up", C.c_float * 3),
                ("z_near", C.c_float), ("z_far", C.c_float),
                ("light_dir", C.c_float * 3), ("ambient", C.c_float), ("diffuse", C.c_float),
                ("ground_enabled", C.c_uint32), ("ground_cell", C.c_float), ("ground_grey", C.c_float * 2),
                ("background_rgb", C.c_float * 3)]


class DistractorDesc(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("seed", C.c_uint64),
                ("scale_lo", C.c_float), ("scale_hi", C.c_float), ("offset_lo", C.c_float), ("offset_hi", C.c_float),
                ("d_video", C.c_void_p), ("n_frames", C.c_uint32), ("alpha", C.c_float),
                ("d_env_offset", C.c_void_p), ("n_videos", C.c_uint32), ("d_env_video", C.c_void_p)]


class SkeletonDesc(C.Structure):
    _fields_ = [("n_bodies", C.c_uint32), ("n_free", C.c_uint32), ("n_angles", C.c_uint32),
                ("parent", C.c_void_p), ("slot", C.c_void_p), ("anchor", C.c_void_p), ("axis", C.c_void_p),
                ("offset", C.c_void_p)]


class ConvDesc(C.Structure):
    _fields_ = [("in_h", C.c_uint32), ("in_w", C.c_uint32), ("n_stack", C.c_uint32),
                ("c_out", C.c_uint32), ("kernel", C.c_uint32), ("stride", C.c_uint32),
                ("weights", C.c_void_p), ("bias", C.c_void_p), ("relu", C.c_uint32)]


_lib = None
_lib_path = LIB_PATH


def use_library_file(path):
    """Profiling only (bench.py --profile-lib): load another build of the same sources, e.g. one with phase
    clocks compiled in (paper_2502_00021_amd/build.py --define ... --out FILE).  Must be called before the
    library is first used; nothing in the product path calls it, and no environment variable can."""
    global _lib_path
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    _lib_path = os.path.abspath(path)


def lib():
    """Load libpxr.so (built in-tree by __graft_entry__.build / paper_2502_00021_amd.build)."""
    global _lib
    if _lib is None:
        path = _lib_path
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
        try:  # PyTorch's HIP runtime first: a process that loads this library before it finds no device afterwards
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(path)
        vp, u32 = C.c_void_p, C.c_uint32
        L.pxr_create_scene.argtypes = [C.POINTER(SceneDesc), C.POINTER(vp)]
        L.pxr_destroy_scene.argtypes = [vp]
        L.pxr_apply_distractor.argtypes = [vp, C.POINTER(DistractorDesc)]
        L.pxr_render_batch.argtypes = [vp, vp, vp, u32, u32, u32, u32, vp, vp, vp]
        L.pxr_scene_info.argtypes = [vp, vp, vp, vp, vp]
        L.pxr_set_block_threads.argtypes = [vp, u32]
        L.pxr_host_tables.argtypes = [C.POINTER(SceneDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.pxr_set_skeleton.argtypes = [vp, C.POINTER(SkeletonDesc)]
        L.pxr_pose_batch.argtypes = [vp, vp, vp, u32, vp, vp]
        L.pxr_render_batch_kinematic.argtypes = [vp, vp, vp, vp, u32, u32, u32, u32, vp, vp, vp, vp]
        L.pxr_render_batch_kinematic_static.argtypes = [vp, vp, vp, vp, u32, u32, u32, u32, vp, vp, vp]
        L.pxr_render_batch_kinematic_static.restype = C.c_int
        L.pxr_conv_create.argtypes = [C.POINTER(ConvDesc), C.POINTER(vp)]
        L.pxr_conv_destroy.argtypes = [vp]
        L.pxr_conv_forward.argtypes = [vp, vp, u32, vp, vp]
        L.pxr_conv_info.argtypes = [vp, vp, vp, vp, vp, vp]
        L.pxr_conv_set_tuning.argtypes = [vp, u32, u32]
        for name in ("pxr_conv_create", "pxr_conv_destroy", "pxr_conv_forward", "pxr_conv_info", "pxr_conv_set_tuning"):
            getattr(L, name).restype = C.c_int
        L.pxr_pipeline_create.argtypes = [vp, vp, u32, C.POINTER(vp)]
        L.pxr_pipeline_destroy.argtypes = [vp]
        L.pxr_pipeline_step.argtypes = [vp, vp, vp, u32, u32, u32, vp, vp, vp]
        for name in ("pxr_pipeline_create", "pxr_pipeline_destroy", "pxr_pipeline_step"):
            getattr(L, name).restype = C.c_int
        L.pxr_selftest_arithmetic.argtypes = [vp]
        L.pxr_selftest_arithmetic.restype = C.c_int
        L.pxr_measure_peaks.argtypes = [vp, vp, vp, vp, vp]
        L.pxr_measure_peaks.restype = C.c_int
        L.pxr_last_error.restype = C.c_char_p
        for name in ("pxr_create_scene", "pxr_destroy_scene", "pxr_apply_distractor", "pxr_render_batch",
                     "pxr_scene_info", "pxr_set_block_threads", "pxr_host_tables", "pxr_set_skeleton",
                     "pxr_pose_batch", "pxr_render_batch_kinematic"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc):
    if rc != OK:
        raise PxrError(rc, lib().pxr_last_error().decode())


def make_scene_desc(desc):
    """Plain-dict scene description (see workloads.default_scene) -> (SceneDesc, keep-alive list)."""
    bodies = desc["bodies"]
    arr = (BodyDesc * max(1, len(bodies)))()
    keep = [arr]
    for i, b in enumerate(bodies):
        arr[i].type = KINDS[b["kind"]] if isinstance(b["kind"], str) else int(b["kind"])
        arr[i].shape = (C.c_float * 4)(*b["shape"])
        arr[i].rgb = (C.c_float * 3)(*b["rgb"])
        arr[i].n_lon = int(b["n_lon"])
        arr[i].n_lat = int(b.get("n_lat", 0))
        if b.get("verts") is not None:  # caller-supplied mesh
            v = np.ascontiguousarray(b["verts"], dtype=np.float32).reshape(-1, 3)
            t = np.ascontiguousarray(b["tris"], dtype=np.uint32).reshape(-1, 3)
            keep += [v, t]
            arr[i].mesh_verts, arr[i].mesh_tris = v.ctypes.data, t.ctypes.data
            arr[i].n_mesh_verts, arr[i].n_mesh_tris = v.shape[0], t.shape[0]
            if b.get("mul") is not None:
                m = np.ascontiguousarray(b["mul"], dtype=np.float32)
                assert m.shape == (t.shape[0],)
                keep.append(m)
                arr[i].mesh_tri_mul = m.ctypes.data
    d = SceneDesc()
    d.width, d.height = int(desc["width"]), int(desc["height"])
    d.n_bodies, d.root_body = len(bodies), int(desc["root_body"])
    d.bodies = C.cast(arr, C.POINTER(BodyDesc))
    d.fov_y_deg = desc["fov_y_deg"]
    d.cam_offset = (C.c_float * 3)(*desc["cam_offset"])
    d.cam_up = (C.c_float * 3)(*desc["cam_up"])
    d.z_near, d.z_far = desc["z_near"], desc["z_far"]
    d.light_dir = (C.c_float * 3)(*desc["light_dir"])
    d.ambient, d.diffuse = desc["ambient"], desc["diffuse"]
    d.ground_enabled = 1 if desc["ground_enabled"] else 0
    d.ground_cell = desc["ground_cell"]
    d.ground_grey = (C.c_float * 2)(*desc["ground_grey"])
    d.background_rgb = (C.c_float * 3)(*desc["background_rgb"])
    return d, keep


def host_tables(desc):
    """pxr_host_tables: the scene builder's tables as numpy arrays (no device needed)."""
    d, keep = make_scene_desc(desc)
    nv, nt, npair = C.c_uint32(), C.c_uint32(), C.c_uint32()
    _check(lib().pxr_host_tables(C.byref(d), C.byref(nv), C.byref(nt), None, None, None, None, None,
                                 C.byref(npair), None))
    V, T, P = nv.value, nt.value, npair.value
    pt = np.empty((P, 3), np.uint32)
    vt = np.empty((V, 4), np.float32)
    ti = np.empty((T, 2), np.uint32)
    ts = np.empty((T, 4), np.float32)
    cxcy = np.empty(d.width + d.height, np.float32)
    consts = np.empty(16, np.float32)
    _check(lib().pxr_host_tables(C.byref(d), None, None, vt.ctypes.data, ti.ctypes.data, ts.ctypes.data,
                                 cxcy.ctypes.data, consts.ctypes.data, None, pt.ctypes.data))
    del keep
    code = vt[:, 3].copy().view(np.uint32)
    return dict(V=V, T=T, uverts=np.concatenate([vt[:, :3], ((code & 3).astype(np.float32) - 1.0)[:, None]], axis=1),
                vert_body=code >> 2,
                tris=np.stack([ti[:, 0] & 0xFFFF, ti[:, 0] >> 16, ti[:, 1] & 0xFFFF], axis=1).astype(np.uint32),
                tri_body=ti[:, 1] >> 16, normals=ts[:, :3].copy(), mul=ts[:, 3].copy(),
                cx=cxcy[:d.width].copy(), cy=cxcy[d.width:].copy(),
                Rv=consts[:9].reshape(3, 3).copy(), f=float(consts[9]), gs=consts[10:12].copy(), l=consts[12:15].copy(),
                lds_bytes=int(consts[15]),
                pair_quads=np.stack([pt[:, 0] & 0xFFFF, pt[:, 0] >> 16, pt[:, 1] & 0xFFFF, pt[:, 1] >> 16], axis=1),
                pair_tris=np.stack([pt[:, 2] & 0xFFFF, pt[:, 2] >> 16], axis=1))


class Scene:
    """Owns one pxr_scene handle.  Tensors passed to render_batch must live on the scene's GPU."""

    def __init__(self, desc):
        d, keep = make_scene_desc(desc)
        h = C.c_void_p()
        _check(lib().pxr_create_scene(C.byref(d), C.byref(h)))
        del keep
        self._h = h
        self.W, self.H, self.K = d.width, d.height, d.n_bodies
        self._bound = []  # keeps bound distractor tensors alive
        self._skel = None  # (n_free, n_angles) of the bound skeleton

    def close(self):
        if getattr(self, "_h", None):
            _check(lib().pxr_destroy_scene(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def info(self):
        v, t, l, b = C.c_uint32(), C.c_uint32(), C.c_uint32(), C.c_uint32()
        _check(lib().pxr_scene_info(self._h, C.byref(v), C.byref(t), C.byref(l), C.byref(b)))
        return dict(n_verts=v.value, n_tris=t.value, lds_bytes=l.value, block_threads=b.value)

    def set_block_threads(self, n):
        _check(lib().pxr_set_block_threads(self._h, int(n)))

    def apply_distractor(self, d=None):
        """d: None / {"mode": "none"} to unbind, or a dict as produced by the workload generators,
        with `video` / `env_offset` given as CUDA uint8 / int32 tensors."""
        self._bound = []
        if d is None or d.get("mode", "none") == "none":
            _check(lib().pxr_apply_distractor(self._h, None))
            return
        unknown = set(d) - {"mode", "seed", "scale", "offset", "video", "alpha", "env_offset", "env_video"}
        if unknown:  # (a misspelt key would silently leave its default in place)
            raise ValueError(f"unknown distractor keys: {sorted(unknown)}")
        s = DistractorDesc()
        s.mode = MODES[d["mode"]]
        s.seed = int(d.get("seed", 0))
        s.scale_lo, s.scale_hi = d.get("scale", (1.0, 1.0))
        s.offset_lo, s.offset_hi = d.get("offset", (0.0, 0.0))
        if d["mode"] == "video":
            v = d["video"]
            assert v.is_cuda and v.is_contiguous() and v.dtype.itemsize == 1 and tuple(v.shape[-3:]) == (self.H, self.W, 3)
            s.d_video = v.data_ptr()
            if v.dim() == 5:  # a set of clips [n_videos, n_frames, H, W, 3]
                s.n_videos, s.n_frames = v.shape[0], v.shape[1]
                ev = d.get("env_video")
                if ev is not None:
                    assert ev.is_cuda and ev.is_contiguous() and ev.dtype.itemsize == 4
                    s.d_env_video = ev.data_ptr()
                    self._bound.append(ev)
            else:
                assert v.dim() == 4
                s.n_frames = v.shape[0]
            s.alpha = float(d.get("alpha", 0.5))
            self._bound.append(v)
            eo = d.get("env_offset")
            if eo is not None:
                assert eo.is_cuda and eo.is_contiguous() and eo.dtype.itemsize == 4
                s.d_env_offset = eo.data_ptr()
                self._bound.append(eo)
        _check(lib().pxr_apply_distractor(self._h, C.byref(s)))

    def render_batch(self, poses, shapes=None, step0=0, env0=0, frames=None, ids=None, want_ids=False, stream=None):
        """poses: CUDA float32 [B,S,K,7]; shapes: CUDA float32 [B,K,4] or None.
        Returns (frames uint8 [B,S,H,W,3], ids int32-typed uint32 bits [B,S,H,W] or None); enqueue only."""
        import torch
        assert poses.is_cuda and poses.dtype == torch.float32 and poses.is_contiguous()
        B, S = int(poses.shape[0]), int(poses.shape[1])
        assert tuple(poses.shape) == (B, S, self.K, 7), tuple(poses.shape)
        if shapes is not None:
            assert shapes.is_cuda and shapes.dtype == torch.float32 and shapes.is_contiguous()
            assert tuple(shapes.shape) == (B, self.K, 4)
        if frames is None:
            frames = torch.empty((B, S, self.H, self.W, 3), dtype=torch.uint8, device=poses.device)
        else:
            assert frames.is_cuda and frames.is_contiguous() and frames.dtype == torch.uint8
            assert tuple(frames.shape) == (B, S, self.H, self.W, 3)
        if ids is None and want_ids:
            ids = torch.empty((B, S, self.H, self.W), dtype=torch.int32, device=poses.device)
        if ids is not None:
            assert ids.is_cuda and ids.is_contiguous() and ids.dtype == torch.int32
            assert tuple(ids.shape) == (B, S, self.H, self.W)
        if stream is None:
            stream = torch.cuda.current_stream(poses.device).cuda_stream
        _check(lib().pxr_render_batch(self._h, poses.data_ptr(), None if shapes is None else shapes.data_ptr(),
                                      B, S, int(step0), int(env0), frames.data_ptr(),
                                      None if ids is None else ids.data_ptr(), C.c_void_p(stream)))
        return frames, ids


    # ---- kinematics stage

    def set_skeleton(self, skel, n_free, n_angles):
        """skel: dict(parent, slot, anchor, axis, offset) of length-K host arrays (workloads._skeleton), or None."""
        if skel is None:
            _check(lib().pxr_set_skeleton(self._h, None))
            self._skel = None
            return
        d, keep = make_skeleton_desc(skel, n_free, n_angles)
        _check(lib().pxr_set_skeleton(self._h, C.byref(d)))
        del keep
        self._skel = (int(n_free), int(n_angles))

    def _fk_args(self, free_poses, angles):
        import torch
        if self._skel is None:
            raise PxrError(ERR_INVALID_ARG, "no skeleton bound (Scene.set_skeleton)")
        F, J = self._skel
        lead = tuple(free_poses.shape[:-2]) if F else tuple(angles.shape[:-1])
        n = int(np.prod(lead))
        if F:
            assert free_poses.is_cuda and free_poses.dtype == torch.float32 and free_poses.is_contiguous()
            assert tuple(free_poses.shape) == lead + (F, 7), tuple(free_poses.shape)
        if J:
            assert angles.is_cuda and angles.dtype == torch.float32 and angles.is_contiguous()
            assert tuple(angles.shape) == lead + (J,), tuple(angles.shape)
        dev = free_poses.device if F else angles.device
        return lead, n, dev, (free_poses.data_ptr() if F else None), (angles.data_ptr() if J else None)

    def pose_batch(self, free_poses, angles, poses=None, stream=None):
        """free_poses: CUDA float32 [..., F, 7]; angles: CUDA float32 [..., J] -> poses [..., K, 7]; enqueue only."""
        import torch
        lead, n, dev, pf, pa = self._fk_args(free_poses, angles)
        if poses is None:
            poses = torch.empty(lead + (self.K, 7), dtype=torch.float32, device=dev)
        else:
            assert poses.is_cuda and poses.is_contiguous() and poses.dtype == torch.float32
            assert tuple(poses.shape) == lead + (self.K, 7)
        if stream is None:
            stream = torch.cuda.current_stream(dev).cuda_stream
        _check(lib().pxr_pose_batch(self._h, pf, pa, n, poses.data_ptr(), C.c_void_p(stream)))
        return poses

    def render_batch_kinematic(self, free_poses, angles, shapes=None, step0=0, env0=0, poses=None, frames=None,
                               want_ids=False, stream=None):
        """free_poses [B,S,F,7], angles [B,S,J] -> (frames, ids or None, poses [B,S,K,7]); enqueue only."""
        import torch
        lead, n, dev, pf, pa = self._fk_args(free_poses, angles)
        B, S = lead
        if poses is None:
            poses = torch.empty((B, S, self.K, 7), dtype=torch.float32, device=dev)
        if frames is None:
            frames = torch.empty((B, S, self.H, self.W, 3), dtype=torch.uint8, device=dev)
        assert poses.is_contiguous() and tuple(poses.shape) == (B, S, self.K, 7) and poses.dtype == torch.float32
        assert frames.is_contiguous() and tuple(frames.shape) == (B, S, self.H, self.W, 3) and frames.dtype == torch.uint8
        if shapes is not None:
            assert shapes.is_cuda and shapes.dtype == torch.float32 and shapes.is_contiguous()
            assert tuple(shapes.shape) == (B, self.K, 4)
        ids = torch.empty((B, S, self.H, self.W), dtype=torch.int32, device=dev) if want_ids else None
        if stream is None:
            stream = torch.cuda.current_stream(dev).cuda_stream
        _check(lib().pxr_render_batch_kinematic(self._h, pf, pa, None if shapes is None else shapes.data_ptr(), B, S,
                                                int(step0), int(env0), poses.data_ptr(), frames.data_ptr(),
                                                None if ids is None else ids.data_ptr(), C.c_void_p(stream)))
        return frames, ids, poses


    def render_batch_kinematic_static(self, free_poses, angles, shapes=None, step0=0, env0=0, frames=None, ids=None,
                                      stream=None):
        """pxr_render_batch_kinematic_static: like render_batch_kinematic, the poses staying in the library's own
        static device buffer.  `frames` (and `ids`, if wanted) must be given: this call allocates nothing."""
        import torch
        lead, n, dev, pf, pa = self._fk_args(free_poses, angles)
        B, S = lead
        assert frames is not None and frames.is_cuda and frames.is_contiguous() and frames.dtype == torch.uint8
        assert tuple(frames.shape) == (B, S, self.H, self.W, 3)
        if ids is not None:
            assert ids.is_cuda and ids.is_contiguous() and ids.dtype == torch.int32 and tuple(ids.shape) == (B, S, self.H, self.W)
        if shapes is not None:
            assert shapes.is_cuda and shapes.dtype == torch.float32 and shapes.is_contiguous()
            assert tuple(shapes.shape) == (B, self.K, 4)
        if stream is None:
            stream = torch.cuda.current_stream(dev).cuda_stream
        _check(lib().pxr_render_batch_kinematic_static(self._h, pf, pa, None if shapes is None else shapes.data_ptr(), B, S,
                                                       int(step0), int(env0), frames.data_ptr(),
                                                       None if ids is None else ids.data_ptr(), C.c_void_p(stream)))
        return frames, ids


class Conv:
    """Owns one pxr_conv handle: the policy's first convolutional layer (3x3, stride 2, 32 channels) on the frame stack."""

    def __init__(self, in_h, in_w, n_stack, weights, bias, relu=True, c_out=32, kernel=3, stride=2):
        w = np.ascontiguousarray(weights, dtype=np.float32)
        b = np.ascontiguousarray(bias, dtype=np.float32)
        assert w.shape == (kernel, kernel, 3 * n_stack, c_out) and b.shape == (c_out,), (w.shape, b.shape)
        d = ConvDesc()
        d.in_h, d.in_w, d.n_stack = int(in_h), int(in_w), int(n_stack)
        d.c_out, d.kernel, d.stride = int(c_out), int(kernel), int(stride)
        d.weights, d.bias, d.relu = w.ctypes.data, b.ctypes.data, 1 if relu else 0
        h = C.c_void_p()
        _check(lib().pxr_conv_create(C.byref(d), C.byref(h)))
        self._h = h
        self.H, self.W, self.S, self.C = int(in_h), int(in_w), int(n_stack), int(c_out)
        i = self.info()
        self.Ho, self.Wo = i["out_h"], i["out_w"]

    def close(self):
        if getattr(self, "_h", None):
            _check(lib().pxr_conv_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def info(self):
        v = [C.c_uint32() for _ in range(5)]
        _check(lib().pxr_conv_info(self._h, *[C.byref(x) for x in v]))
        return dict(zip(("out_h", "out_w", "band_rows", "lds_bytes", "n_groups"), (x.value for x in v)))

    def set_tuning(self, band_rows=0, n_groups=0):
        _check(lib().pxr_conv_set_tuning(self._h, int(band_rows), int(n_groups)))

    def forward(self, frames, out=None, stream=None):
        """frames: CUDA uint8 [B,S,H,W,3] -> CUDA bfloat16 [B,Ho,Wo,32]; enqueue only."""
        import torch
        assert frames.is_cuda and frames.dtype == torch.uint8 and frames.is_contiguous()
        B = int(frames.shape[0])
        assert tuple(frames.shape) == (B, self.S, self.H, self.W, 3), tuple(frames.shape)
        if out is None:
            out = torch.empty((B, self.Ho, self.Wo, self.C), dtype=torch.bfloat16, device=frames.device)
        else:
            assert out.is_cuda and out.is_contiguous() and out.dtype == torch.bfloat16
            assert tuple(out.shape) == (B, self.Ho, self.Wo, self.C)
        if stream is None:
            stream = torch.cuda.current_stream(frames.device).cuda_stream
        _check(lib().pxr_conv_forward(self._h, frames.data_ptr(), B, out.data_ptr(), C.c_void_p(stream)))
        return out


class Pipeline:
    """Owns one pxr_pipeline handle: render + conv layer per step, chunk c's layer beside chunk c + 1's render."""

    def __init__(self, scene, conv, n_chunks=4):
        h = C.c_void_p()
        _check(lib().pxr_pipeline_create(scene._h, conv._h, int(n_chunks), C.byref(h)))
        self._h, self.scene, self.conv = h, scene, conv

    def close(self):
        if getattr(self, "_h", None):
            _check(lib().pxr_pipeline_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, poses, shapes, frames, features, step0=0, env0=0, stream=None):
        """poses [B,S,K,7], shapes [B,K,4] or None -> frames [B,S,H,W,3] uint8, features [B,Ho,Wo,32] bf16 (both given)."""
        import torch
        sc, cv = self.scene, self.conv
        B = int(poses.shape[0])
        assert poses.is_cuda and poses.dtype == torch.float32 and poses.is_contiguous() and tuple(poses.shape) == (B, cv.S, sc.K, 7)
        if shapes is not None:
            assert shapes.is_cuda and shapes.dtype == torch.float32 and shapes.is_contiguous() and tuple(shapes.shape) == (B, sc.K, 4)
        assert frames.is_cuda and frames.is_contiguous() and frames.dtype == torch.uint8 and tuple(frames.shape) == (B, cv.S, sc.H, sc.W, 3)
        assert features.is_cuda and features.is_contiguous() and features.dtype == torch.bfloat16
        assert tuple(features.shape) == (B, cv.Ho, cv.Wo, cv.C)
        if stream is None:
            stream = torch.cuda.current_stream(poses.device).cuda_stream
        _check(lib().pxr_pipeline_step(self._h, poses.data_ptr(), None if shapes is None else shapes.data_ptr(), B,
                                       int(step0), int(env0), frames.data_ptr(), features.data_ptr(), C.c_void_p(stream)))
        return frames, features


def make_skeleton_desc(skel, n_free, n_angles):
    """dict(parent, slot, anchor, axis, offset) -> (SkeletonDesc, keep-alive list)."""
    parent = np.ascontiguousarray(skel["parent"], dtype=np.int32)
    slot = np.ascontiguousarray(skel["slot"], dtype=np.int32)
    arrs = [np.ascontiguousarray(skel[k], dtype=np.float32).reshape(-1) for k in ("anchor", "axis", "offset")]
    K = parent.shape[0]
    assert slot.shape == (K,) and all(a.shape == (K * 3,) for a in arrs)
    d = SkeletonDesc()
    d.n_bodies, d.n_free, d.n_angles = K, int(n_free), int(n_angles)
    d.parent, d.slot = parent.ctypes.data, slot.ctypes.data
    d.anchor, d.axis, d.offset = (a.ctypes.data for a in arrs)
    return d, [parent, slot] + arrs


def selftest_arithmetic():
    """pxr_selftest_arithmetic: dict(recip_mismatches, floor_mismatches, recip_checked, floor_checked) on the current device."""
    c = (C.c_uint64 * 4)()
    _check(lib().pxr_selftest_arithmetic(c))
    return dict(recip_mismatches=int(c[0]), floor_mismatches=int(c[1]), recip_checked=int(c[2]), floor_checked=int(c[3]))


def measure_peaks():
    """pxr_measure_peaks: dict(fma_tlaneops, imad_tlaneops, copy_gbs, read_gbs, write_gbs) measured on the current device."""
    v = [C.c_double() for _ in range(5)]
    _check(lib().pxr_measure_peaks(*[C.byref(x) for x in v]))
    return dict(zip(("fma_tlaneops", "imad_tlaneops", "copy_gbs", "read_gbs", "write_gbs"), (x.value for x in v)))


def ids_to_numpy(ids):
    """int32 CUDA tensor holding uint32 id bits -> numpy uint32."""
    return ids.cpu().numpy().view(np.uint32)
