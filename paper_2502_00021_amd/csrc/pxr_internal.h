// Internal layout shared by the host-side scene builder and the HIP kernels of
// libpxr.  Nothing here is visible through the C ABI (include/pxr.h).
#ifndef PXR_INTERNAL_H
#define PXR_INTERNAL_H

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "pxr.h"

namespace pxr {

// Sentinel stored in the snapped-X array for a vertex that is unusable (outside the
// guard band, or a non-finite depth); any triangle touching it is dropped.
constexpr int32_t kRejectedX = INT32_MIN;
// Sentinel for a vertex behind the near plane: its triangles are clipped against the plane in the
// raster phase.  (Snapped coordinates stay within +-2^22, so both sentinels sort below every real one.)
constexpr int32_t kBehindX = INT32_MIN + 1;

// Raster bins by the number of pixel centres in a surviving triangle's clamped bounding box:
//   tiny  <= kTinyMaxPixels   one lane
//   small <= kSmallMaxPixels  a team of 2^kSmallLanesLog2 lanes, rows dealt round-robin
//   large otherwise           a whole wavefront, one row per lane (also: triangles to be clipped)
// What is balanced here is the longest chain in the raster phase, not the instruction count: one lane
// walking a 12-pixel triangle holds up its whole workgroup at the next barrier.
constexpr uint32_t kTinyMaxPixels = 3;
constexpr uint32_t kSmallMaxPixels = 128;
constexpr uint32_t kSmallLanesLog2 = 2;
constexpr uint32_t kNoTriangle = 0xFFFFu;
// Banded frames: a band picks the triangles that touch its rows out of the frame's bins in rounds of one per lane;
// a round's lists therefore never hold more than the largest workgroup has lanes.
constexpr uint32_t kBandListEntries = 1024;
// ... which pays from this many bands on; with fewer, every band walks all bins (lds_blist == 0).
constexpr uint32_t kBandListsFrom = 6;

// Per-body record kept in LDS for the duration of one frame (floats).
//   [0..8]  M  = view rotation * body rotation, row-major
//   [9..11] t  = body origin in view space
//   [12..14] lb = light direction in the body frame
//   [15]    pad
//   [16..19] shape (a,b,c,h)
//   [20..22] rgb, [23] pad
constexpr uint32_t kBodyStride = 24;

// Everything the kernel needs that is constant for a scene.  Passed by value
// as the kernel argument (lands in SGPRs / scalar loads).
struct SceneConsts {
    // camera rows (right, up, forward), eye offset, focal length in pixels
    float Rt[3], Up[3], Fw[3], off[3];
    float f, halfW, halfH, z_near, z_far;
    // light, ground, background
    float l[3], ambient, diffuse;
    float cell, gs[2], bg[3];
    uint32_t ground_on;
    uint32_t checker_short_form;  // cell == 1 and z_far <= 2^64: no division, and ground points of a frame whose eye is no NaN are no NaNs
    // sizes
    uint32_t W, H, npix, K, root, V, T, P;  // P = entries of the pair table (on the device: padded to a multiple of 64)
    uint32_t band_rows;                     // rows of the frame held by the LDS key buffer at a time
    uint32_t first_band_rows;               // rows of the first band (<= band_rows); later bands have band_rows
    uint32_t magicW;  // ceil(2^32 / W): p / W == mulhi(p, magicW) for every pixel index p < 512 * W
    // device tables
    const float* vtmpl;       // [V][4]  ux,uy,uz, bits = (LDS byte address of the body's record)<<2 | s as a 2-bit signed number
                              //         (the host-side table holds body<<2 | (s+1))
    const uint32_t* tri_idx;  // [T][2]  v0 | v1<<16 ,  v2 | body<<16
    const float* tri_shade;   // [T][4]  unit normal (body frame), colour multiplier
    const uint32_t* pair_tbl; // [P][4]  a0 | a1<<16 , a2 | a3<<16 , triA | triB<<16 , 0 (a_i = LDS byte address of the cell
                              //         code of vertex q_i; the host-side table holds q_i itself): two triangles sharing the
                              //         edge q0-q2, or one triangle (q3 = q2, triB = kNoTriangle); the device copy ends with padding entries
    //         (no triangles; the four addresses are that of the word after the last vertex's code, which holds code 0)
    const float* body_const;  // [K][8]  shape a,b,c,h ; rgb r,g,b,0   then, on the device, [4][3]: Rt, Up, Fw, l
    const float* cxcy;        // [W+H]   pixel-centre ray slopes
    // LDS carve-up (byte offsets into the dynamic segment)
    // the lds_keys region first holds the per-vertex cell codes (u32[V]) and the candidate list (u16[T])
    uint32_t lds_keys, lds_vxy, lds_vd, lds_body, lds_list, lds_large, lds_cxcy, lds_rows, lds_misc, lds_total;
    uint32_t lds_blist, lds_blist2;  // banded frames: one band round's lists (kBandListEntries u16 each)
    uint32_t lds_vlut;  // video-blend tables (kVideoTableBytes), or 0 if the frame's LDS has no room for them
};

// Video distractor: for each of the five colours that can lie under the clip (background r, g, b; the two ground
// greys) the blended, quantised byte for every clip byte: [5][256] bytes, rebuilt per frame in LDS.
constexpr uint32_t kVideoTableBytes = 9 * 256;  // background r, g, b; first grey x 3; second grey x 3

// Distractor state bound by pxr_apply_distractor.
struct DistractConsts {
    uint32_t mode;
    uint32_t seed_lo, seed_hi;
    float scale_lo, scale_span, offset_lo, offset_span;
    const uint8_t* video;
    uint32_t n_frames;
    float alpha;
    const uint32_t* env_offset;
    uint32_t n_videos;          // >= 1
    const uint32_t* env_video;  // [B] or null
};

// Skeleton bound by pxr_set_skeleton (device tables live in their own allocation).
struct SkeletonConsts {
    uint32_t K, J, F;        // bodies, hinge angles per frame, free poses per frame
    const int32_t* parent;   // [K]  -1 = free body
    const int32_t* slot;     // [K]  free: index of its pose; hinged: index of its angle, -1 = rigid
    const float* hinge;      // [K][9]  anchor (parent frame), unit axis, body centre relative to the hinge (body frame)
};

// Host-side result of tessellation + camera derivation.
struct HostScene {
    SceneConsts c{};
    std::vector<float> vtmpl;
    std::vector<uint32_t> tri_idx;
    std::vector<float> tri_shade;
    std::vector<uint32_t> pair_tbl;
    std::vector<float> body_const;
    std::vector<float> cxcy;
};

// scene.cpp: validates `desc`, fills `hs` (device pointers and LDS offsets are
// left for the caller).  Returns a PXR_* code and a message on failure.
int build_host_scene(const pxr_scene_desc& desc, HostScene& hs, std::string& err);

// render.hip: enqueue one batch.  `block_threads` in {256,512,768,1024}.
int launch_render(const SceneConsts& sc, const DistractConsts& dc, const float* d_poses, const float* d_shapes,
                  uint32_t n_frames, uint32_t S, uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids,
                  uint32_t block_threads, void* stream, std::string& err);

// render.hip: raise the dynamic-LDS limit of every kernel instantiation on the current device (the caller sees
// to it that this runs once per device).
int prepare_kernels(std::string& err);

// Frame consumer (first convolutional layer of the policy), bound by pxr_conv_create.
// 3x3 kernel, stride 2, 32 output channels; the frame stack is the channel axis.
struct ConvConsts {
    uint32_t H, W, S;        // input frames [S,H,W,3] per environment
    uint32_t Ho, Wo;         // output size
    uint32_t tiles_x;        // 32-pixel tiles per output row
    uint32_t tiles_magic;    // ceil(2^16 / tiles_x): task / tiles_x == (task * tiles_magic) >> 16 for task < 2^13
    uint32_t band_rows;      // output rows per work item
    uint32_t bands;          // work items per environment
    uint32_t rows_in;        // input rows held in LDS per frame = 2 * band_rows + 1
    uint32_t relu;
    const uint32_t* wtab;    // [3S][64 lanes][4] the A operands of the matrix instruction, bf16 pairs
    const float* bias;       // [32]
};

// api.cpp: record the calling thread's last error and return `code`.
int set_error(int code, const std::string& msg);

// conv.hip
uint32_t conv_lds_bytes(const ConvConsts& cc);
uint32_t conv_max_quads();  // 12-byte input quads (4 pixels) one work item may hold: S * rows_in * W / 4
int prepare_conv_kernels(std::string& err);
int launch_conv(const ConvConsts& cc, const uint8_t* d_frames, uint32_t B, uint16_t* d_out, uint32_t n_groups,
                void* stream, std::string& err);

// peaks.hip: sustained fp32-FMA and 24-bit integer multiply-add rates (T lane-operations/s) and the
// read+write bandwidth of a plain 1 GiB copy and of 2 GiB read-only / write-only streams (GB/s) on the current device.
int measure_peaks(double* fma_tlaneops, double* imad_tlaneops, double* copy_gbs, double* read_gbs, double* write_gbs,
                  std::string& err);

// selftest.hip: the render kernel's arithmetic shortcuts against the plain forms over every float
// (counts: reciprocal mismatches, floor-convert mismatches, patterns looked at by each check).
int selftest_arithmetic(unsigned long long counts[4], std::string& err);

// kinematics.hip: joint angles -> poses, one lane per frame.
uint32_t fk_lds_bytes(const SkeletonConsts& sk);
int prepare_fk_kernel(std::string& err);
int launch_fk(const SkeletonConsts& sk, const float* d_free_poses, const float* d_angles, uint32_t n_frames,
              float* d_poses, void* stream, std::string& err);

// pipeline.cpp works through these (api.cpp / conv_api.cpp own the handles' layouts).
constexpr uint32_t kMaxPipelineChunks = 16;
void scene_shape(const pxr_scene* s, uint32_t* K, uint32_t* H, uint32_t* W);
void conv_shape(const pxr_conv* c, uint32_t* H, uint32_t* W, uint32_t* S, uint32_t* Ho, uint32_t* Wo);
// Environments [e0, e0 + n) of a batch whose buffers start at the given pointers (arguments as pxr_render_batch /
// pxr_conv_forward, whose checks they repeat; per-environment distractor arrays are indexed by position in the batch).
int render_envs(pxr_scene* s, const float* d_poses, const float* d_shapes, uint32_t e0, uint32_t n, uint32_t S,
                uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids, void* stream, std::string& err);
int conv_envs(pxr_conv* c, const uint8_t* d_frames, uint32_t e0, uint32_t n, uint16_t* d_out, void* stream, std::string& err);

// static_scratch.hip: this device's copy of the library's file-scope pose buffer (looked up on the first call
// per device, cached afterwards) and its size.  Allocates nothing.
int static_pose_scratch(float** out, size_t* capacity_bytes, std::string& err);

}  // namespace pxr

#endif
