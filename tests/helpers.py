"""Small numpy-only helpers shared by the tests (double-precision reference geometry)."""
import numpy as np

from paper_2502_00021_amd import workloads as wl


def quat_to_mat(q):
    """Textbook unit-quaternion (w,x,y,z) rotation matrix, float64."""
    w, x, y, z = [float(v) for v in q]
    return np.array([[1 - 2 * (y * y + z * z), 2 * (x * y - w * z), 2 * (x * z + w * y)],
                     [2 * (x * y + w * z), 1 - 2 * (x * x + z * z), 2 * (y * z - w * x)],
                     [2 * (x * z - w * y), 2 * (y * z + w * x), 1 - 2 * (x * x + y * y)]])


def look_at(desc):
    """Rows (right, up, forward) of the view rotation and focal length in pixels, float64."""
    off = np.array(desc["cam_offset"], dtype=np.float64)
    up = np.array(desc["cam_up"], dtype=np.float64)
    fw = -off / np.linalg.norm(off)
    rt = np.cross(fw, up)
    rt /= np.linalg.norm(rt)
    upv = np.cross(rt, fw)
    f = (desc["height"] / 2.0) / np.tan(np.radians(desc["fov_y_deg"]) / 2.0)
    return np.stack([rt, upv, fw]), f


def local_positions(mesh, shapes):
    """Posed-shape local vertex positions (float64) from the unit template: (a*ux, b*uy, c*uz + s*h)."""
    uv = mesh["uverts"].astype(np.float64)
    sh = np.asarray(shapes, dtype=np.float64)[mesh["vert_body"]]
    return np.stack([sh[:, 0] * uv[:, 0], sh[:, 1] * uv[:, 1], sh[:, 2] * uv[:, 2] + uv[:, 3] * sh[:, 3]], axis=1)


def world_positions(mesh, shapes, poses):
    """World-space vertex positions (float64) for one frame; poses [K,7]."""
    loc = local_positions(mesh, shapes)
    out = np.empty_like(loc)
    for b in range(len(poses)):
        m = mesh["vert_body"] == b
        R = quat_to_mat(poses[b, 3:7])
        out[m] = loc[m] @ R.T + np.asarray(poses[b, :3], dtype=np.float64)
    return out


def one_body_scene(body, W=32, H=32, **over):
    d = wl.default_scene(W, H, [body])
    d.update(over)
    return d


def pose_row(pos, quat=(1.0, 0.0, 0.0, 0.0)):
    return np.array([*pos, *quat], dtype=np.float32)
