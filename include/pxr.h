/*
 * pxr — batched pixel-observation renderer for one AMD MI355X (gfx950).
 *
 * C ABI of the hot path that PixelBrax (arXiv 2502.00021) moves onto the
 * accelerator: for each of B parallel environments and each of S steps, turn
 * the simulator's rigid-body poses into one small RGB observation without the
 * frame ever leaving the device (paper section 1), optionally with a colour or
 * a video distractor fused into the renderer (paper section 2) and with all
 * randomness drawn from an explicit seeded generator (paper sections 1-2).
 *
 * All functions return a PXR_* status code, never throw or abort across the
 * ABI, and leave out-parameters untouched on error.  pxr_last_error() gives a
 * human-readable reason for the last failure on the calling thread.
 *
 * Pointers named d_* are DEVICE pointers owned by the caller; everything else
 * is host memory.  The library owns only the pxr_scene and the device-side
 * constants it uploads at creation.
 */
#ifndef PXR_H
#define PXR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pxr_scene pxr_scene; /* opaque, owned by the library */

enum { PXR_OK = 0, PXR_ERR_INVALID_ARG = 1, PXR_ERR_UNSUPPORTED = 2, PXR_ERR_OOM = 3, PXR_ERR_DEVICE = 4 };
enum { PXR_CAPSULE = 0, PXR_SPHERE = 1, PXR_BOX = 2, PXR_MESH = 3 };
enum { PXR_DISTRACT_NONE = 0, PXR_DISTRACT_COLOR = 1, PXR_DISTRACT_VIDEO = 2 };

/* Winning-id values that are not triangles. */
#define PXR_ID_GROUND 0xFFFFFFFEu
#define PXR_ID_BG     0xFFFFFFFFu

/* One rigid body = one primitive, tessellated once at scene creation.
 *   shape: capsule (r,r,r,h): radius r, half-length h of the segment along local +Z
 *          sphere  (r,r,r,0)
 *          box     (ex,ey,ez,0): half-extents
 *          The posed local vertex is (shape[0]*ux, shape[1]*uy, shape[2]*uz + s*shape[3]) for the
 *          unit-shape template vertex (ux,uy,uz) with cap selector s.
 *   n_lon, n_lat: capsule/sphere: longitudes, latitude steps PER HEMISPHERE
 *          (capsule 4*n_lon*n_lat triangles, sphere 2*n_lon*(2*n_lat-1));
 *          box: n_lon = cells per face edge (12*n_lon^2 triangles, checker
 *          colour multiplier 1 / 0.5 per cell), n_lat ignored.
 *   PXR_MESH (the paper names mesh rendering as its renderer's next step): the caller's own triangle mesh.
 *          mesh_verts [n_mesh_verts*3] body-frame positions, used as the template as they are (selector 0,
 *          scaled per axis by shape[0..2], shape[3] ignored); mesh_tris [n_mesh_tris*3] indices into them,
 *          counter-clockwise seen from outside (back faces are culled); mesh_tri_mul [n_mesh_tris] colour
 *          multiplier per triangle, or NULL = 1.  Host arrays, copied at scene creation; ignored for the
 *          other types.  A triangle's normal is the unit cross product of its unscaled vertices (zero for
 *          a triangle without area: it is shaded with the ambient term only). */
typedef struct {
    uint32_t type;
    float shape[4];
    float rgb[3];
    uint32_t n_lon, n_lat;
    const float* mesh_verts;
    const uint32_t* mesh_tris;
    const float* mesh_tri_mul;
    uint32_t n_mesh_verts, n_mesh_tris;
} pxr_body_desc;

/* Scene = what is common to all environments: image size, bodies, camera rig,
 * light, ground, background.  The camera sits at (root body position +
 * cam_offset) in WORLD axes and looks at the root body; pinhole, fov_y_deg
 * vertical field of view.  light_dir points TOWARD the light.  The ground is
 * the plane z = 0 with a two-grey checkerboard of ground_cell metres. */
typedef struct {
    uint32_t width, height, n_bodies, root_body;
    const pxr_body_desc* bodies; /* host, borrowed for the call only */
    float fov_y_deg, cam_offset[3], cam_up[3], z_near, z_far;
    float light_dir[3], ambient, diffuse;
    uint32_t ground_enabled;
    float ground_cell, ground_grey[2];
    float background_rgb[3];
} pxr_scene_desc;

/* Distractor state (paper section 2: the colour kind or the video kind, mutually exclusive).
 *   COLOR: per (env, step) and per channel, scale ~ U[scale_lo,scale_hi) and
 *          offset ~ U[offset_lo,offset_hi) from the counter-based generator
 *          keyed by (seed, env, step); every pixel becomes clamp(c*scale+offset, 0, 1).
 *   VIDEO: d_video is a device-resident uint8 [n_frames,H,W,3] clip; env e at
 *          step t shows frame (env_offset[e] + t) mod n_frames, alpha-blended
 *          onto pixels whose winner is the ground or the background.
 *          d_env_offset: device uint32 [B] (indexed by the env's position in
 *          the batch), or NULL = drawn from the generator.  With n_videos > 1
 *          every environment plays one clip of a set (paper section 2: each
 *          environment gets a clip picked at random), chosen by d_env_video or
 *          drawn from the generator.  All buffers are caller-owned and must stay alive while bound. */
typedef struct {
    uint32_t mode;
    uint64_t seed;
    float scale_lo, scale_hi, offset_lo, offset_hi;
    const uint8_t* d_video;
    uint32_t n_frames;
    float alpha;
    const uint32_t* d_env_offset;
    uint32_t n_videos;            /* VIDEO: 0 or 1 = one clip; > 1: d_video is [n_videos,n_frames,H,W,3] */
    const uint32_t* d_env_video;  /* VIDEO, n_videos > 1: device uint32 [B], the clip of each environment
                                     (values >= n_videos are reduced modulo n_videos), or NULL = drawn */
} pxr_distractor_desc;

/* Build a scene on the current HIP device: validate, tessellate, derive the
 * camera constants, upload (one allocation, one synchronous copy).  Host only,
 * not on the hot path.  (Paper section 1: an environment is a set of rigid bodies seen by a camera; the
 * paper gives no geometry, camera or lighting model, so primitives, tessellation, the root-tracking pinhole
 * camera and the flat Lambert-plus-ambient light are this library's reading of "rendered from the
 * simulator's state".)
 * Errors: INVALID_ARG (null pointer, root_body out of range, unknown body
 * type, non-finite or non-positive parameter, a colour (rgb, ground_grey, background_rgb) outside [0,1], a
 * negative mesh colour multiplier, degenerate camera, mesh index out of range or non-finite mesh vertex);
 * UNSUPPORTED (width or height outside [8,512], n_bodies outside [1,64], more
 * than 65535 vertices or triangles, tessellation counts outside [3,64]x[1,32]
 * (box [1,16]), or a frame that does not fit the 160 KB of LDS of one
 * compute unit); OOM; DEVICE. */
int pxr_create_scene(const pxr_scene_desc* desc, pxr_scene** out);

/* Free the scene and its device constants (the counterpart of pxr_create_scene; paper section 1: the
 * renderer's state lives on the device for as long as the environments do).  The caller must have
 * synchronised every stream that still renders from it.  NULL is accepted. */
int pxr_destroy_scene(pxr_scene* s);

/* Bind (or with d == NULL / mode NONE, unbind) the distractor that later
 * pxr_render_batch calls fuse into their final per-pixel pass (paper section
 * 2: distractors live inside the renderer).  Host only; launches nothing.
 * Errors: INVALID_ARG (unknown mode, non-finite range, VIDEO with null
 * d_video or n_frames == 0 or alpha outside [0,1]). */
int pxr_apply_distractor(pxr_scene* s, const pxr_distractor_desc* d);

/* Render B environments x S steps = B*S frames (the hot path; paper section 1:
 * one pixel observation per parallel environment per step, on the device).
 *   d_poses  [B,S,K,7] fp32: position xyz, unit quaternion wxyz (body -> world)
 *   d_shapes [B,K,4]   fp32 per-environment shapes, or NULL = the scene's
 *   step0    step index of s = 0 (frame s of the call is step step0 + s; it
 *            keys the generator and selects the video frame)
 *   env0     global index of the batch's first environment (keys the generator,
 *            so a shard renders the same bytes as the whole batch would)
 *   d_frames [B,S,H,W,3] uint8, R,G,B, row-major, written completely
 *   d_ids    [B,S,H,W] uint32 winning triangle id / PXR_ID_GROUND / PXR_ID_BG,
 *            or NULL
 *   hip_stream  hipStream_t to enqueue on; NULL = the default stream
 * Only enqueues and returns: no synchronisation, no host<->device copy, no
 * allocation.  Pose VALUES are not validated.  A triangle with corners on both sides of the near plane
 * z_near is clipped against it (the part in front is drawn); one wholly behind it is not drawn; a vertex
 * in front that projects more than 16384 pixels from the image centre, or a non-finite one, removes its
 * triangles from the frame.
 * Alignment: d_poses, d_frames 4 bytes; d_shapes (16-byte records), d_ids 16 bytes.
 * Errors: INVALID_ARG (null scene/poses/frames, B*S == 0, B*S > 2^31-1,
 * step0 + S or env0 + B overflow, misaligned buffer); DEVICE (launch failure). */
int pxr_render_batch(pxr_scene* s, const float* d_poses, const float* d_shapes, uint32_t B, uint32_t S,
                     uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids, void* hip_stream);

/* Kinematic tree of the scene's bodies, for callers whose simulator state is joint angles rather than
 * body poses (the paper's loop keeps that state on the device, section 1; this stage turns it into the
 * renderer's input there).  All arrays are host memory, copied by pxr_set_skeleton.
 *   parent[k]  -1: body k is free, its pose is free pose number slot[k] (0 <= slot[k] < n_free), copied
 *              verbatim; otherwise body k hangs on body parent[k] < k by a hinge
 *   slot[k]    hinged body: index of its angle (0 <= slot[k] < n_angles), or -1 = rigidly attached (angle 0)
 *   anchor[k]  hinge position in the parent's frame; axis[k] unit hinge axis (same in both frames);
 *   offset[k]  body centre relative to the hinge, in the body's own frame   (each [n_bodies*3])
 * Pose of a hinged body: q = q_parent (x) (cos(a/2), sin(a/2) axis);
 *   p = (p_parent + R(q_parent) anchor) + R(q) offset,  fp32, R as in the vertex stage.  sin and cos of a/2 are
 *   within 1.25 * 2^-24 of the true values for |a| <= 65536 rad; an angle beyond that or a non-finite one makes
 *   the body's pose, and those of its descendants, NaN (their triangles are not drawn). */
typedef struct {
    uint32_t n_bodies, n_free, n_angles;
    const int32_t* parent;
    const int32_t* slot;
    const float* anchor;
    const float* axis;
    const float* offset;
} pxr_skeleton_desc;

/* Bind (or with k == NULL remove) the scene's skeleton.  Host only; one small allocation and upload.  The
 * caller must have synchronised streams still using the previous skeleton.
 * Errors: INVALID_ARG (null array, n_bodies != the scene's, parent[k] >= k, slot out of range, non-finite
 * entry); UNSUPPORTED (the 64 frames a wavefront poses at a time do not fit the 160 KB of LDS:
 * (7*n_bodies + 7*n_free + n_angles) * 260 bytes); OOM; DEVICE. */
int pxr_set_skeleton(pxr_scene* s, const pxr_skeleton_desc* k);

/* Forward kinematics for N frames: d_free_poses [N,n_free,7] and d_angles [N,n_angles] (may be NULL when
 * the count is 0) -> d_poses [N,n_bodies,7] (xyz, wxyz), all fp32 device buffers, 4-byte aligned.  One kernel,
 * one lane per frame; enqueue only.  Errors: INVALID_ARG (no skeleton bound, null or misaligned buffer,
 * N == 0); DEVICE. */
int pxr_pose_batch(pxr_scene* s, const float* d_free_poses, const float* d_angles, uint32_t n_frames,
                   float* d_poses, void* hip_stream);

/* pxr_pose_batch over B*S frames followed by pxr_render_batch on the same stream: joint angles in, frames
 * out, nothing crossing the host.  d_poses [B,S,n_bodies,7] is caller-provided and receives the poses (a
 * learner usually wants them as well); the other arguments are those of the two calls. */
int pxr_render_batch_kinematic(pxr_scene* s, const float* d_free_poses, const float* d_angles, const float* d_shapes,
                               uint32_t B, uint32_t S, uint32_t step0, uint32_t env0, float* d_poses,
                               uint8_t* d_frames, uint32_t* d_ids, void* hip_stream);

/* pxr_render_batch_kinematic for callers that cannot allocate device memory or provide a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The poses between the two
 * kernels live in a 32 MiB buffer that is part of the library's image on each GPU (held until the process
 * ends) instead of in d_poses; they are not returned.  The call allocates and frees nothing and only enqueues.
 * Calls on one GPU share that buffer: two calls whose kernels may overlap (different streams without an
 * ordering between them) race; calls on one stream, or ordered by events, are safe.  Nothing carries over
 * from one call to the next.
 * Errors: those of pxr_render_batch_kinematic, and UNSUPPORTED when B * S * n_bodies * 28 bytes exceed
 * 32 MiB (33 554 432); DEVICE if the buffer's address cannot be obtained. */
int pxr_render_batch_kinematic_static(pxr_scene* s, const float* d_free_poses, const float* d_angles,
                                      const float* d_shapes, uint32_t B, uint32_t S, uint32_t step0, uint32_t env0,
                                      uint8_t* d_frames, uint32_t* d_ids, void* hip_stream);

/* ---- frame consumer: the policy's first convolutional layer on the frame stack ----
 * The paper's throughput loop ends every environment step with a forward pass through one convolutional
 * layer on the observations (section 2); it gives no hyper-parameters.  Built here: 3x3 kernel, stride 2, no
 * padding, 32 output channels, the S frames of an environment stacked on the channel axis (channel 3s + c),
 * inputs scaled by 1/255:
 *   out[b,oy,ox,o] = act(bias[o] + sum_{ky,kx,s,c} frames[b,s,2oy+ky,2ox+kx,c]/255 * bf16(w[ky,kx,3s+c,o]))
 * weights rounded to bfloat16 (nearest even) at creation, products and sums in fp32 on the matrix cores,
 * result = fma(sum, 1/255, bias), optional ReLU, rounded to bfloat16 (nearest even). */
typedef struct pxr_conv pxr_conv; /* opaque, owned by the library */
typedef struct {
    uint32_t in_h, in_w, n_stack;  /* frames [B,n_stack,in_h,in_w,3] uint8 */
    uint32_t c_out, kernel, stride; /* must be 32, 3, 2 */
    const float* weights;          /* host [3][3][3*n_stack][32] (height, width, in, out), copied */
    const float* bias;             /* host [32], copied */
    uint32_t relu;                 /* 0 = linear output */
} pxr_conv_desc;

/* Host only.  Errors: INVALID_ARG (null, non-finite weight or bias); UNSUPPORTED (other layer shapes,
 * n_stack outside [1,4], in_h outside [3,512], in_w outside [4,256] or not a multiple of 4); OOM; DEVICE. */
int pxr_conv_create(const pxr_conv_desc* desc, pxr_conv** out);
/* Free a layer made by pxr_conv_create (same passage).  NULL accepted; synchronise streams still using it first. */
int pxr_conv_destroy(pxr_conv* c);

/* d_frames [B,n_stack,in_h,in_w,3] uint8 (what pxr_render_batch writes for S = n_stack) ->
 * d_out [B,out_h,out_w,32] bfloat16 bit patterns, out_h = (in_h-3)/2+1, out_w = (in_w-3)/2+1.
 * Device buffers owned by the caller, d_frames 4-byte and d_out 16-byte aligned.  One kernel, enqueue only.
 * Errors: INVALID_ARG (null, B == 0 or too large, misaligned); DEVICE. */
int pxr_conv_forward(pxr_conv* c, const uint8_t* d_frames, uint32_t B, uint16_t* d_out, void* hip_stream);

/* Facts about a layer (no passage of the paper): output size, output rows per work item, LDS bytes per
 * workgroup, persistent workgroups per launch.  Any pointer may be NULL.  Errors: INVALID_ARG (null layer). */
int pxr_conv_info(const pxr_conv* c, uint32_t* out_h, uint32_t* out_w, uint32_t* band_rows, uint32_t* lds_bytes,
                  uint32_t* n_groups);

/* Tuning knob for benchmarks: output rows per work item and workgroups per launch (0 = default).  The
 * output does not depend on it. */
int pxr_conv_set_tuning(pxr_conv* c, uint32_t band_rows, uint32_t n_groups);

/* ---- renderer and consumer as one step ----
 * The paper's throughput loop (section 2) renders every environment and then runs the conv layer on the
 * frames, every step.  The renderer is bound by vector-ALU issue and the layer by HBM, so this call runs them
 * side by side: the batch is cut into n_chunks runs of environments, chunk c is rendered on the caller's stream
 * and its conv layer follows on a second stream (created here, default priority) while chunk c + 1 is rendered;
 * ordering is by events only, and the caller's stream is made to wait for the last layer before the call
 * returns (enqueue only, no host synchronisation, no allocation).  Frames and features are byte for byte those
 * of pxr_render_batch followed by pxr_conv_forward.  n_chunks = 1 is that serial order. */
typedef struct pxr_pipeline pxr_pipeline; /* opaque, owned by the library; borrows the scene and the layer */

/* Host only: one stream and n_chunks + 1 events.  The layer's input size must be the scene's frame size; its
 * n_stack is the S of every step.  Errors: INVALID_ARG (null, n_chunks outside [1,16], sizes differ); OOM; DEVICE. */
int pxr_pipeline_create(pxr_scene* s, pxr_conv* c, uint32_t n_chunks, pxr_pipeline** out);
/* Waits for the second stream, then frees it and the events; scene and layer stay the caller's.  NULL accepted. */
int pxr_pipeline_destroy(pxr_pipeline* p);
/* d_poses [B,S,K,7], d_shapes [B,K,4] or NULL, d_frames [B,S,H,W,3] (written), d_features [B,Ho,Wo,32] bf16
 * (written): arguments, alignment and errors as for pxr_render_batch and pxr_conv_forward.  Steps issued on
 * one pipeline must be ordered among themselves (one stream, or events): they share the second stream. */
int pxr_pipeline_step(pxr_pipeline* p, const float* d_poses, const float* d_shapes, uint32_t B, uint32_t step0,
                      uint32_t env0, uint8_t* d_frames, uint16_t* d_features, void* hip_stream);

/* Scene facts for callers and tests (sizes of what pxr_create_scene built; no passage of the paper): total
 * template vertices and triangles, dynamic LDS bytes per frame workgroup, threads per workgroup.  Any out
 * pointer may be NULL.  Errors: INVALID_ARG (null scene). */
int pxr_scene_info(const pxr_scene* s, uint32_t* n_verts, uint32_t* n_tris, uint32_t* lds_bytes,
                   uint32_t* block_threads);

/* Override the threads per frame workgroup (256, 512, 768 or 1024); 0 restores the
 * default.  A tuning knob for benchmarks; output does not depend on it. */
int pxr_set_block_threads(pxr_scene* s, uint32_t threads);

/* Measurement aid (synchronous, allocates 2 GiB for the duration of the call): the rates this GPU sustains
 * on a dependent-free fp32 FMA loop and on a 24-bit integer multiply-add loop (both in T lane-operations/s,
 * 32 waves per compute unit), the read+write bandwidth of a plain 1 GiB device-to-device copy and the
 * bandwidths of a 2 GiB read-only and a 2 GiB write-only stream (GB/s; HBM does not give both directions
 * the same rate).  Lets a roofline fraction be quoted against the machine as it runs.  Any pointer may be
 * NULL.  Errors: OOM, DEVICE. */
int pxr_measure_peaks(double* fma_tlaneops, double* imad_tlaneops, double* copy_gbs, double* read_gbs, double* write_gbs);

/* Verification aid (synchronous, a few tens of milliseconds): the render kernel replaces two operations whose
 * results decide integers by shorter instruction sequences - 1/x by the hardware estimate plus one fused
 * Newton step, (int)floorf(x) by one converting instruction.  This call compares each with the plain form on
 * the current device for EVERY 32-bit pattern in its domain (x in [2^-100, 2^100]; every x that is not NaN)
 * and writes to the host array counts[4]: reciprocal mismatches, floor mismatches, patterns checked by the
 * first and by the second comparison.  Both mismatch counts must be 0 on a device the library supports.
 * Errors: INVALID_ARG (null), OOM, DEVICE. */
int pxr_selftest_arithmetic(uint64_t* counts);

/* Host-only introspection: run the scene builder of pxr_create_scene without
 * touching a device and copy out its tables, so that the tessellation and the
 * camera constants can be checked on a machine without a GPU.  Any output
 * pointer may be NULL.  Same validation errors as pxr_create_scene.
 *   vtmpl     [V*4] ux,uy,uz and a word holding body<<2 | (s+1)
 *   tri_idx   [T*2] v0 | v1<<16 ,  v2 | body<<16
 *   tri_shade [T*4] unit normal in the body frame, colour multiplier
 *   cxcy      [W+H] ray slopes of the pixel-centre columns, then rows
 *   consts    [16]  right[3], up[3], forward[3], focal, ground shade[2], light[3], LDS bytes
 *   pair_tbl  [P*3] binning table: q0 | q1<<16, q2 | q3<<16, triA | triB<<16 (two triangles sharing the
 *             edge q0-q2; a lone triangle has q3 = q2 and triB = 0xFFFF); P is returned in n_pairs */
int pxr_host_tables(const pxr_scene_desc* desc, uint32_t* n_verts, uint32_t* n_tris, float* vtmpl, uint32_t* tri_idx,
                    float* tri_shade, float* cxcy, float* consts, uint32_t* n_pairs, uint32_t* pair_tbl);

/* Reason for the last failure on this thread; valid until the next call on it.  (Error reporting of this
 * interface; no passage of the paper.) */
const char* pxr_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
