/*
 * orc — the CPU oracle of the batched pixel-observation renderer.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded
 * rasterizer that defines what the GPU library must compute.  It is linked by
 * nothing in the product path: only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg load it.  It shares no source, header, table
 * or helper with the HIP library.
 *
 * The paper (PixelBrax, sections 1 and 2) fixes only WHAT is produced: one
 * small RGB observation per parallel environment per step, rendered from the
 * simulator's rigid-body poses on the accelerator, optionally with a colour
 * distractor (the whole frame's colour bias changes at every step) or a video
 * distractor (frame t of a device-resident video is overlaid at step t), all
 * randomness drawn from an explicit seeded generator.  It says nothing about
 * geometry, camera, raster rules or precision; those conventions are this
 * build's reading and are written out, step by step, in orc.cpp.
 *
 * Pins (tests/test_oracle_*.py): mesh counts, closedness, orientation and
 * volume; camera orthonormality and centre projection; axis-aligned quad
 * pixel counts and watertightness; convex cover count; front set == back set;
 * exact rational point-in-triangle; permutation invariance; analytic and
 * Moller-Trumbore ray casts; horizon row; shade extremes; RNG bijectivity and
 * statistics; distractor identities; kinematics against float64 quaternion algebra (an independent
 * numpy implementation) and closed-form hinge geometry.
 * The generator reproduces the published Philox-4x32-10 known-answer vectors
 * (tests/golden/philox4x32_10_kat.txt).
 */
#ifndef ORC_H
#define ORC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_ID_GROUND 0xFFFFFFFEu
#define ORC_ID_BG     0xFFFFFFFFu

/* primitive kinds */
#define ORC_CAPSULE 0u
#define ORC_SPHERE  1u
#define ORC_BOX     2u
#define ORC_MESH    3u

/* distractor modes (paper section 2: "color" or "video") */
#define ORC_DIS_NONE  0u
#define ORC_DIS_COLOR 1u
#define ORC_DIS_VIDEO 2u

typedef struct orc_scene orc_scene;

/* Scene parameters, all host memory, all copied.
 *   kinds[K], shapes[K*4] (a,b,c,h), rgbs[K*3], n_lon[K], n_lat[K]
 *   cam[9]    = fov_y_deg, offset xyz, up xyz, z_near, z_far
 *   light[5]  = direction-toward-light xyz, ambient, diffuse
 *   ground[4] = enabled (0/1), cell size, grey0, grey1
 *   bg[3]     = background rgb
 * Returns NULL on invalid input. */
orc_scene* orc_scene_create(uint32_t width, uint32_t height, uint32_t n_bodies, uint32_t root_body,
                            const uint32_t* kinds, const float* shapes, const float* rgbs,
                            const uint32_t* n_lon, const uint32_t* n_lat,
                            const float* cam, const float* light, const float* ground, const float* bg);
/* The same, with caller-supplied triangle meshes for the bodies of kind ORC_MESH (the paper names mesh
 * rendering as the renderer's next step).  mesh_nv[K], mesh_nt[K]: vertex / triangle counts per body (0 for
 * the other kinds); mesh_verts / mesh_tris / mesh_mul: the meshes of the ORC_MESH bodies concatenated in body
 * order ([sum nv][3] body-frame positions, [sum nt][3] indices local to the body's own vertices,
 * counter-clockwise seen from outside, [sum nt] colour multipliers or NULL = 1).  A mesh vertex is posed
 * like any template vertex (scaled per axis by shape[0..2]); a triangle's normal is the unit cross product
 * of its unscaled vertices. */
orc_scene* orc_scene_create_meshes(uint32_t width, uint32_t height, uint32_t n_bodies, uint32_t root_body,
                                   const uint32_t* kinds, const float* shapes, const float* rgbs,
                                   const uint32_t* n_lon, const uint32_t* n_lat,
                                   const float* cam, const float* light, const float* ground, const float* bg,
                                   const uint32_t* mesh_nv, const uint32_t* mesh_nt, const float* mesh_verts,
                                   const uint32_t* mesh_tris, const float* mesh_mul);
void orc_scene_destroy(orc_scene* s);

/* total template vertices / triangles */
void orc_scene_counts(const orc_scene* s, uint32_t* n_verts, uint32_t* n_tris);

/* Template mesh: unit vertices (ux,uy,uz,s)[V*4], index triples [T*3] (global
 * vertex ids), unit normals [T*3] (body frame), colour multiplier [T], owning
 * body of each triangle [T] and of each vertex [V].  Any pointer may be NULL. */
void orc_scene_mesh(const orc_scene* s, float* uverts, uint32_t* tris, float* normals, float* mul,
                    uint32_t* tri_body, uint32_t* vert_body);

/* Camera constants: Rv[9] (rows right, up, forward), f, cx[W], cy[H], gs[2], l[3]. */
void orc_scene_camera(const orc_scene* s, float* Rv, float* f, float* cx, float* cy, float* gs, float* l);

/* Vertex stage for ONE frame: poses[K*7] = (px,py,pz,qw,qx,qy,qz) per body,
 * shapes[K*4] or NULL (scene shapes).  Writes snapped X[V], Y[V] (8 sub-pixel
 * bits), reversed depth D[V] and rejected[V] (0 = usable; 2 = behind the near
 * plane, its triangles are clipped by orc_render; 1 = outside the guard band or
 * non-finite, its triangles are dropped; X,Y,D are 0 unless usable).  eye[3]
 * (may be NULL) receives the camera position. */
void orc_vertex_stage(const orc_scene* s, const float* poses, const float* shapes,
                      int32_t* X, int32_t* Y, float* D, uint8_t* rejected, float* eye);

/* Raster + z-test of an arbitrary snapped triangle soup (no scene needed).
 *   order: permutation of [0,n_tris) giving the submission order, or NULL
 *   cull:  0 = keep front faces (the renderer's rule), 1 = keep back faces
 *          instead, 2 = full-image candidate loop instead of the bbox loop
 *          (front faces)
 * Outputs (each may be NULL): ids[H*W] winning triangle id or ORC_ID_BG,
 * depth_bits[H*W] float bits of the winning depth (0 where background),
 * cover[H*W] number of kept triangles covering each pixel centre. */
void orc_raster(uint32_t width, uint32_t height, uint32_t n_verts, const int32_t* X, const int32_t* Y,
                const float* D, const uint8_t* rejected, uint32_t n_tris, const uint32_t* tris,
                const uint32_t* order, uint32_t cull, uint32_t* ids, uint32_t* depth_bits, uint32_t* cover);

/* Distractor parameters for orc_render. */
typedef struct {
    uint32_t mode;
    uint64_t seed;
    float scale_lo, scale_hi, offset_lo, offset_hi; /* colour mode */
    const uint8_t* video;                           /* video mode: [n_frames,H,W,3], host */
    uint32_t n_frames;
    float alpha;
    const uint32_t* env_offset;                     /* [B] or NULL -> drawn from the generator */
    uint32_t n_videos;                              /* 0 or 1: one clip; > 1: video is [n_videos,n_frames,H,W,3] */
    const uint32_t* env_video;                      /* [B] clip of each environment, or NULL -> drawn (stream 3) */
} orc_distractor;

/* Full path: poses[B,S,K,7], shapes[B,K,4] or NULL, frames[B,S,H,W,3] out,
 * ids[B,S,H,W] out or NULL, depth_bits[B,S,H,W] out or NULL.  env0 is the
 * global index of the first environment (the generator is keyed by global
 * environment index).  order = optional triangle submission order.
 * A triangle with corners on both sides of the near plane is clipped against it in view space (corners in
 * front kept, crossing edges cut from the corner in front towards the one behind, 3 or 4 corners
 * re-projected, snapped and rastered as one or two triangles under the same id); orc_raster, which sees only
 * snapped coordinates, drops such triangles. */
int orc_render(const orc_scene* s, const float* poses, const float* shapes, uint32_t B, uint32_t S,
               uint32_t step0, uint32_t env0, const orc_distractor* dis, const uint32_t* order,
               uint8_t* frames, uint32_t* ids, uint32_t* depth_bits);

/* Forward kinematics for ONE frame (producer stage in front of the renderer: the paper's loop keeps the
 * simulator state on the device, section 1; here joint angles become body poses without leaving it).
 * Body k is either free (parent[k] < 0: its pose is free_poses[slot[k]], copied verbatim) or hangs on
 * body parent[k] < k by a hinge: anchor[k] = hinge position in the parent's frame, axis[k] = unit hinge
 * axis, offset[k] = body centre relative to the hinge in the body's own frame, angle = angles[slot[k]]
 * (slot[k] < 0: rigidly attached, angle 0).  sin and cos of the half angle are the C library's in double,
 * rounded once to fp32 (NaN for an angle beyond +-65536 rad or non-finite); the quaternion and position
 * algebra is fp32 in a fixed order (orc.cpp, section F).
 * out_poses[K*7] = px,py,pz,qw,qx,qy,qz.  Returns non-zero on a malformed skeleton. */
int orc_fk(uint32_t n_bodies, const int32_t* parent, const int32_t* slot, const float* anchor, const float* axis,
           const float* offset, const float* free_poses, const float* angles, float* out_poses);

/* Counter-based generator: 10 rounds of the 4x32 multiply/xor network on
 * counter (c0..c3) under the 64-bit key `seed`; out[4]. */
void orc_philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t* out);
/* 24-bit uniform in [0,1) from one 32-bit word. */
float orc_u01(uint32_t x);

#ifdef __cplusplus
}
#endif
#endif
