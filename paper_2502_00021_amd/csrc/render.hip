// The hot path of libpxr: one HIP kernel, one workgroup per frame
// (= environment x step), the whole frame resident in LDS from the posed
// vertices to the packed uint8 store.  gfx950 only.
//
// What it renders is what PixelBrax (arXiv 2502.00021, sections 1-2) asks of
// its renderer: a small RGB observation per parallel environment per step,
// built on the device from the simulator's body poses, with the colour / video
// distractors applied inside the renderer and all randomness coming from a
// seeded counter-based generator.
//
// Phases of one workgroup (barriers between them):
//   0  clear the pixel keys, load per-body transforms          (LDS)
//   1  instancing: template vertex -> view space -> snapped fixed point
//   2  binning: per triangle cull + pixel-range test; survivors are compacted
//      wave-wide (ballot + mbcnt) into a "one lane" bin and a "whole wave" bin
//   3  raster: integer edge functions, top-left rule, float reversed depth,
//      64-bit LDS atomic max on (depth bits << 32 | ~triangle id)
//   4  resolve: ground ray, id -> flat Lambert colour, distractor, uint8 pack,
//      coalesced 12-byte stores
//
// Floating point is written with explicit fmaf and compiled with
// -ffp-contract=off: the order of operations is part of the output contract
// (coverage is decided by integers derived from these floats).

#include <hip/hip_runtime.h>

#include "pxr_internal.h"

namespace pxr {
namespace {

typedef unsigned long long u64;

__device__ __forceinline__ float dot3(float a0, float a1, float a2, float b0, float b1, float b2) {
    return __builtin_fmaf(a0, b0, __builtin_fmaf(a1, b1, a2 * b2));
}

__device__ __forceinline__ int imin3(int a, int b, int c) { return min(a, min(b, c)); }
__device__ __forceinline__ int imax3(int a, int b, int c) { return max(a, max(b, c)); }

// Workgroups are dealt round-robin to the 8 XCDs.  Renumber them so that each
// XCD works on one contiguous run of frames: neighbouring frames share pose
// cache lines and (video mode) neighbouring clip frames in that XCD's L2.
__device__ __forceinline__ uint32_t frame_of_block(uint32_t bid, uint32_t nb) {
    const uint32_t q = nb >> 3, r = nb & 7u, xcd = bid & 7u, idx = bid >> 3;
    return xcd < r ? xcd * (q + 1) + idx : r * (q + 1) + (xcd - r) * q + idx;
}

// ---------------------------------------------------------------- generator
// 10 rounds of the 4x32 multiply / xor counter network, key = 64-bit seed,
// counter = (env, step, stream, 0).
__device__ __forceinline__ void counter_rng(uint32_t k0, uint32_t k1, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0;
        c1 = lo1;
        c2 = n2;
        c3 = lo0;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}
__device__ __forceinline__ float unit_float(uint32_t x) { return (float)(x >> 8) * 5.9604644775390625e-08f; }

// ---------------------------------------------------------------- raster helpers

struct TriSetup {
    int ax, ay, bx, by, cx, cy;  // screen order a = v0, b = v2, c = v1
    float Da, dDb, dDc;
    int i0, i1, j0, j1;
};

// Edge pq is "top-left" when it points up, or is horizontal pointing right
// (y grows downwards): pixels exactly on it belong to the triangle.
__device__ __forceinline__ int edge_bias(int dx, int dy) { return (dy < 0 || (dy == 0 && dx > 0)) ? 0 : -1; }

__device__ __forceinline__ void z_test(u64* keys, uint32_t pix, float depth, uint32_t tri) {
    const u64 key = ((u64)__float_as_uint(depth) << 32) | (u64)(0xFFFFFFFFu - tri);
    atomicMax(&keys[pix], key);
}

// One lane walks the (at most kSmallMaxPixels) pixel centres of a small
// triangle.  All differences fit in 16 bits, so 24-bit multiplies are exact.
__device__ __forceinline__ void raster_small(const TriSetup& s, uint32_t tri, uint32_t W, u64* keys) {
    const int dx_ab = s.bx - s.ax, dy_ab = s.by - s.ay;
    const int dx_bc = s.cx - s.bx, dy_bc = s.cy - s.by;
    const int dx_ca = s.ax - s.cx, dy_ca = s.ay - s.cy;
    const int A2 = __mul24(dx_ab, s.cy - s.ay) - __mul24(dy_ab, s.cx - s.ax);
    const float invA = 1.0f / (float)A2;
    const int b_ab = edge_bias(dx_ab, dy_ab), b_bc = edge_bias(dx_bc, dy_bc), b_ca = edge_bias(dx_ca, dy_ca);
    const int px0 = (s.i0 << 8) + 128, py0 = (s.j0 << 8) + 128;
    int r_ab = __mul24(dx_ab, py0 - s.ay) - __mul24(dy_ab, px0 - s.ax);
    int r_bc = __mul24(dx_bc, py0 - s.by) - __mul24(dy_bc, px0 - s.bx);
    int r_ca = __mul24(dx_ca, py0 - s.cy) - __mul24(dy_ca, px0 - s.cx);
    for (int j = s.j0; j <= s.j1; ++j) {
        int e_ab = r_ab, e_bc = r_bc, e_ca = r_ca;
        uint32_t pix = (uint32_t)j * W + (uint32_t)s.i0;
        for (int i = s.i0; i <= s.i1; ++i, ++pix) {
            if (((e_ab + b_ab) | (e_bc + b_bc) | (e_ca + b_ca)) >= 0) {
                const float beta = (float)e_ca * invA, gamma = (float)e_ab * invA;
                z_test(keys, pix, __builtin_fmaf(beta, s.dDb, __builtin_fmaf(gamma, s.dDc, s.Da)), tri);
            }
            e_ab -= dy_ab << 8;
            e_bc -= dy_bc << 8;
            e_ca -= dy_ca << 8;
        }
        r_ab += dx_ab << 8;
        r_bc += dx_bc << 8;
        r_ca += dx_ca << 8;
    }
}

// A whole wavefront sweeps a large triangle in 8x8 pixel tiles, one pixel per
// lane, with 64-bit edge functions (coordinates reach 2^22, products 2^46).
__device__ __forceinline__ void raster_wave(const TriSetup& s, uint32_t tri, uint32_t W, u64* keys, uint32_t lane) {
    typedef long long i64;
    const i64 dx_ab = s.bx - s.ax, dy_ab = s.by - s.ay;
    const i64 dx_bc = s.cx - s.bx, dy_bc = s.cy - s.by;
    const i64 dx_ca = s.ax - s.cx, dy_ca = s.ay - s.cy;
    const i64 A2 = dx_ab * (i64)(s.cy - s.ay) - dy_ab * (i64)(s.cx - s.ax);
    const float invA = 1.0f / (float)A2;
    const i64 b_ab = edge_bias((int)dx_ab, (int)dy_ab), b_bc = edge_bias((int)dx_bc, (int)dy_bc),
              b_ca = edge_bias((int)dx_ca, (int)dy_ca);
    const int li = (int)(lane & 7u), lj = (int)(lane >> 3);
    for (int ty = s.j0 & ~7; ty <= s.j1; ty += 8)
        for (int tx = s.i0 & ~7; tx <= s.i1; tx += 8) {
            const int i = tx + li, j = ty + lj;
            if (i < s.i0 || i > s.i1 || j < s.j0 || j > s.j1) continue;
            const i64 px = (i << 8) + 128, py = (j << 8) + 128;
            const i64 e_ab = dx_ab * (py - s.ay) - dy_ab * (px - s.ax);
            const i64 e_bc = dx_bc * (py - s.by) - dy_bc * (px - s.bx);
            const i64 e_ca = dx_ca * (py - s.cy) - dy_ca * (px - s.cx);
            if (((e_ab + b_ab) | (e_bc + b_bc) | (e_ca + b_ca)) >= 0) {
                const float beta = (float)e_ca * invA, gamma = (float)e_ab * invA;
                z_test(keys, (uint32_t)j * W + (uint32_t)i, __builtin_fmaf(beta, s.dDb, __builtin_fmaf(gamma, s.dDc, s.Da)),
                       tri);
            }
        }
}

// Gather a triangle's snapped vertices and its clamped pixel-centre range.
// Returns false if a vertex was rejected or no pixel centre is inside the
// bounding box.  `small_extent` = both fixed-point extents below 2^15.
__device__ __forceinline__ bool tri_gather(const SceneConsts& sc, const uint32_t* __restrict__ tri_idx, uint32_t t,
                                           const int* vx, const int* vy, TriSetup& s, uint32_t& v0, uint32_t& v1,
                                           uint32_t& v2, bool& small_extent) {
    const uint2 ti = reinterpret_cast<const uint2*>(tri_idx)[t];
    v0 = ti.x & 0xFFFFu;
    v1 = ti.x >> 16;
    v2 = ti.y & 0xFFFFu;
    s.ax = vx[v0];
    s.bx = vx[v2];
    s.cx = vx[v1];
    if (s.ax == kRejectedX || s.bx == kRejectedX || s.cx == kRejectedX) return false;
    s.ay = vy[v0];
    s.by = vy[v2];
    s.cy = vy[v1];
    const int minx = imin3(s.ax, s.bx, s.cx), maxx = imax3(s.ax, s.bx, s.cx);
    const int miny = imin3(s.ay, s.by, s.cy), maxy = imax3(s.ay, s.by, s.cy);
    // pixel centres sit at 256 i + 128: first centre >= min, last centre <= max
    s.i0 = max(0, (minx + 127) >> 8);
    s.i1 = min((int)sc.W - 1, (maxx - 128) >> 8);
    s.j0 = max(0, (miny + 127) >> 8);
    s.j1 = min((int)sc.H - 1, (maxy - 128) >> 8);
    small_extent = ((maxx - minx) | (maxy - miny)) < 32768;
    return s.i0 <= s.i1 && s.j0 <= s.j1;
}

__device__ __forceinline__ void tri_depths(TriSetup& s, const float* vd, uint32_t v0, uint32_t v1, uint32_t v2) {
    s.Da = vd[v0];
    s.dDb = vd[v2] - s.Da;
    s.dDc = vd[v1] - s.Da;
}

// ---------------------------------------------------------------- the kernel

struct FrameUniforms {  // written by thread 0 into LDS, read by all after a barrier
    uint32_t n_small, n_large;
    float scale[3], offs[3];
    uint32_t video_frame;
};

template <int NT, int PX>
__global__ __launch_bounds__(NT) void render_kernel(const SceneConsts sc, const DistractConsts dc,
                                                    const float* __restrict__ poses, const float* __restrict__ shapes,
                                                    uint32_t S, uint32_t step0, uint32_t env0,
                                                    uint8_t* __restrict__ frames, uint32_t* __restrict__ ids) {
    extern __shared__ __align__(16) unsigned char lds[];
    u64* keys = reinterpret_cast<u64*>(lds + sc.lds_keys);
    int* vx = reinterpret_cast<int*>(lds + sc.lds_vx);
    int* vy = reinterpret_cast<int*>(lds + sc.lds_vy);
    float* vd = reinterpret_cast<float*>(lds + sc.lds_vd);
    float* body = reinterpret_cast<float*>(lds + sc.lds_body);
    float* cxcy = reinterpret_cast<float*>(lds + sc.lds_cxcy);
    FrameUniforms* fu = reinterpret_cast<FrameUniforms*>(lds + sc.lds_misc);
    uint16_t* list = reinterpret_cast<uint16_t*>(lds + sc.lds_list);

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t frame = frame_of_block(blockIdx.x, gridDim.x);
    const uint32_t e = frame / S;
    const uint32_t step = step0 + (frame - e * S);
    const uint32_t env = env0 + e;
    const float* pose = poses + (size_t)frame * sc.K * 7;

    // camera position: fixed world-space offset from the root body
    const float eye_x = pose[sc.root * 7 + 0] + sc.off[0];
    const float eye_y = pose[sc.root * 7 + 1] + sc.off[1];
    const float eye_z = pose[sc.root * 7 + 2] + sc.off[2];

    // ---- phase 0: clear keys (0 = background at depth 0), per-body transforms, per-frame draws
    for (uint32_t p = tid; p < sc.npix; p += NT) keys[p] = 0ull;
    for (uint32_t i = tid; i < sc.W + sc.H; i += NT) cxcy[i] = sc.cxcy[i];
    if (tid < sc.K) {
        const float* p = pose + tid * 7;
        const float w = p[3], x = p[4], y = p[5], z = p[6];
        float R[3][3];
        R[0][0] = 1.0f - 2.0f * (y * y + z * z);
        R[0][1] = 2.0f * (x * y - w * z);
        R[0][2] = 2.0f * (x * z + w * y);
        R[1][0] = 2.0f * (x * y + w * z);
        R[1][1] = 1.0f - 2.0f * (x * x + z * z);
        R[1][2] = 2.0f * (y * z - w * x);
        R[2][0] = 2.0f * (x * z - w * y);
        R[2][1] = 2.0f * (y * z + w * x);
        R[2][2] = 1.0f - 2.0f * (x * x + y * y);
        const float dx = p[0] - eye_x, dy = p[1] - eye_y, dz = p[2] - eye_z;
        float* o = body + tid * kBodyStride;
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            o[0 + c] = dot3(sc.Rt[0], sc.Rt[1], sc.Rt[2], R[0][c], R[1][c], R[2][c]);
            o[3 + c] = dot3(sc.Up[0], sc.Up[1], sc.Up[2], R[0][c], R[1][c], R[2][c]);
            o[6 + c] = dot3(sc.Fw[0], sc.Fw[1], sc.Fw[2], R[0][c], R[1][c], R[2][c]);
        }
        o[9] = dot3(sc.Rt[0], sc.Rt[1], sc.Rt[2], dx, dy, dz);
        o[10] = dot3(sc.Up[0], sc.Up[1], sc.Up[2], dx, dy, dz);
        o[11] = dot3(sc.Fw[0], sc.Fw[1], sc.Fw[2], dx, dy, dz);
#pragma unroll
        for (int c = 0; c < 3; ++c) o[12 + c] = dot3(sc.l[0], sc.l[1], sc.l[2], R[0][c], R[1][c], R[2][c]);
        const float* shp = shapes ? shapes + ((size_t)e * sc.K + tid) * 4 : sc.body_const + tid * 8;
#pragma unroll
        for (int c = 0; c < 4; ++c) o[16 + c] = shp[c];
#pragma unroll
        for (int c = 0; c < 3; ++c) o[20 + c] = sc.body_const[tid * 8 + 4 + c];
    }
    if (tid == 0) {
        fu->n_small = 0;
        fu->n_large = 0;
        if (dc.mode == PXR_DISTRACT_COLOR) {
            uint32_t r[4];
            counter_rng(dc.seed_lo, dc.seed_hi, env, step, 0u, 0u, r);
#pragma unroll
            for (int c = 0; c < 3; ++c) fu->scale[c] = __builtin_fmaf(unit_float(r[c]), dc.scale_span, dc.scale_lo);
            counter_rng(dc.seed_lo, dc.seed_hi, env, step, 1u, 0u, r);
#pragma unroll
            for (int c = 0; c < 3; ++c) fu->offs[c] = __builtin_fmaf(unit_float(r[c]), dc.offset_span, dc.offset_lo);
        } else if (dc.mode == PXR_DISTRACT_VIDEO) {
            uint32_t first;
            if (dc.env_offset) {
                first = dc.env_offset[e];
            } else {
                uint32_t r[4];
                counter_rng(dc.seed_lo, dc.seed_hi, env, 0xFFFFFFFFu, 2u, 0u, r);
                first = r[0] % dc.n_frames;
            }
            fu->video_frame = (uint32_t)(((u64)first + (u64)step) % dc.n_frames);
        }
    }
    __syncthreads();

    // ---- phase 1: instancing + projection + snap (one lane per template vertex)
    for (uint32_t v = tid; v < sc.V; v += NT) {
        const float4 tv = reinterpret_cast<const float4*>(sc.vtmpl)[v];
        const uint32_t code = __float_as_uint(tv.w);
        const float* o = body + (code >> 2) * kBodyStride;
        const float sel = (float)((int)(code & 3u) - 1);
        const float lx = o[16] * tv.x;
        const float ly = o[17] * tv.y;
        const float lz = __builtin_fmaf(o[18], tv.z, sel * o[19]);
        const float pvx = __builtin_fmaf(o[0], lx, __builtin_fmaf(o[1], ly, __builtin_fmaf(o[2], lz, o[9])));
        const float pvy = __builtin_fmaf(o[3], lx, __builtin_fmaf(o[4], ly, __builtin_fmaf(o[5], lz, o[10])));
        const float pvz = __builtin_fmaf(o[6], lx, __builtin_fmaf(o[7], ly, __builtin_fmaf(o[8], lz, o[11])));
        const float inv = 1.0f / pvz;
        const float sx = __builtin_fmaf(sc.f, pvx * inv, sc.halfW);
        const float sy = __builtin_fmaf(-sc.f, pvy * inv, sc.halfH);
        const bool ok = (pvz >= sc.z_near) && (__builtin_fabsf(sx) <= 16384.0f) && (__builtin_fabsf(sy) <= 16384.0f);
        int X = kRejectedX, Y = 0;
        if (ok) {
            X = (int)__builtin_floorf(__builtin_fmaf(sx, 256.0f, 0.5f));
            Y = (int)__builtin_floorf(__builtin_fmaf(sy, 256.0f, 0.5f));
        }
        vx[v] = X;
        vy[v] = Y;
        vd[v] = sc.z_near * inv;
    }
    __syncthreads();

    // ---- phase 2: binning.  Uniform trip count so that ballots see whole waves.
    for (uint32_t t0 = 0; t0 < sc.T; t0 += NT) {
        const uint32_t t = t0 + tid;
        bool keep = false, small = false;
        if (t < sc.T) {
            TriSetup s;
            uint32_t v0, v1, v2;
            bool small_extent;
            if (tri_gather(sc, sc.tri_idx, t, vx, vy, s, v0, v1, v2, small_extent)) {
                bool front;
                if (small_extent)
                    front = __mul24(s.bx - s.ax, s.cy - s.ay) > __mul24(s.by - s.ay, s.cx - s.ax);
                else
                    front = (long long)(s.bx - s.ax) * (long long)(s.cy - s.ay) >
                            (long long)(s.by - s.ay) * (long long)(s.cx - s.ax);
                keep = front;
                small = small_extent && (uint32_t)((s.i1 - s.i0 + 1) * (s.j1 - s.j0 + 1)) <= kSmallMaxPixels;
            }
        }
        const u64 m_small = __ballot(keep && small);
        const u64 m_large = __ballot(keep && !small);
        if (m_small) {
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&fu->n_small, (uint32_t)__popcll(m_small));
            base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
            if (keep && small)
                list[base + __builtin_amdgcn_mbcnt_hi((uint32_t)(m_small >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m_small, 0u))] =
                    (uint16_t)t;
        }
        if (m_large) {
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&fu->n_large, (uint32_t)__popcll(m_large));
            base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
            if (keep && !small)
                list[sc.T - 1 - (base + __builtin_amdgcn_mbcnt_hi((uint32_t)(m_large >> 32),
                                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)m_large, 0u)))] =
                    (uint16_t)t;
        }
    }
    __syncthreads();

    // ---- phase 3: raster + z-test into the LDS key buffer
    const uint32_t n_small = fu->n_small, n_large = fu->n_large;
    for (uint32_t k = tid; k < n_small; k += NT) {
        const uint32_t t = list[k];
        TriSetup s;
        uint32_t v0, v1, v2;
        bool small_extent;
        tri_gather(sc, sc.tri_idx, t, vx, vy, s, v0, v1, v2, small_extent);
        tri_depths(s, vd, v0, v1, v2);
        raster_small(s, t, sc.W, keys);
    }
    for (uint32_t k = tid >> 6; k < n_large; k += NT / 64) {
        const uint32_t t = list[sc.T - 1 - k];
        TriSetup s;
        uint32_t v0, v1, v2;
        bool small_extent;
        tri_gather(sc, sc.tri_idx, t, vx, vy, s, v0, v1, v2, small_extent);
        tri_depths(s, vd, v0, v1, v2);
        raster_wave(s, t, sc.W, keys, lane);
    }
    __syncthreads();

    // ---- phase 4: resolve + shade + distractor + pack + store
    const bool ground_ok = sc.ground_on && eye_z > 0.0f;
    const float inv_ez = 1.0f / eye_z;
    const uint32_t mode = dc.mode;
    float scale[3] = {1.0f, 1.0f, 1.0f}, offs[3] = {0.0f, 0.0f, 0.0f};
    const uint8_t* vframe = nullptr;
    if (mode == PXR_DISTRACT_COLOR) {
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            scale[c] = fu->scale[c];
            offs[c] = fu->offs[c];
        }
    } else if (mode == PXR_DISTRACT_VIDEO) {
        vframe = dc.video + (size_t)fu->video_frame * sc.npix * 3;
    }
    uint8_t* out = frames + (size_t)frame * sc.npix * 3;
    uint32_t* out_ids = ids ? ids + (size_t)frame * sc.npix : nullptr;

    for (uint32_t q = tid; q * PX < sc.npix; q += NT) {
        const uint32_t p0 = q * PX;
        uint32_t j = __umulhi(p0, sc.magicW);
        uint32_t i = p0 - j * sc.W;
        uint32_t vid[3] = {0u, 0u, 0u};
        if (PX == 4 && mode == PXR_DISTRACT_VIDEO) {
            const uint32_t* vsrc = reinterpret_cast<const uint32_t*>(vframe) + q * 3;
            vid[0] = vsrc[0];
            vid[1] = vsrc[1];
            vid[2] = vsrc[2];
        }
        uint32_t packed[3] = {0u, 0u, 0u};
        uint32_t idv[PX];
#pragma unroll
        for (int k = 0; k < PX; ++k) {
            const uint32_t p = p0 + k;
            u64 key = keys[p];
            // ground: ray through the pixel centre against z = 0
            const float cxi = cxcy[i], cyj = cxcy[sc.W + j];
            const float dwx = __builtin_fmaf(sc.Rt[0], cxi, __builtin_fmaf(sc.Up[0], cyj, sc.Fw[0]));
            const float dwy = __builtin_fmaf(sc.Rt[1], cxi, __builtin_fmaf(sc.Up[1], cyj, sc.Fw[1]));
            const float dwz = __builtin_fmaf(sc.Rt[2], cxi, __builtin_fmaf(sc.Up[2], cyj, sc.Fw[2]));
            const float ndz = -dwz;
            float tg = 0.0f;
            if (ground_ok && ndz > 0.0f) {
                tg = eye_z / ndz;
                if (tg >= sc.z_near && tg <= sc.z_far) {
                    const float dg = (sc.z_near * ndz) * inv_ez;
                    const u64 gkey = ((u64)__float_as_uint(dg) << 32) | 1ull;
                    key = key > gkey ? key : gkey;
                }
            }
            const uint32_t low = (uint32_t)key;
            float c[3];
            if (low == 0u) {
                c[0] = sc.bg[0];
                c[1] = sc.bg[1];
                c[2] = sc.bg[2];
            } else if (low == 1u) {
                const float wx = __builtin_fmaf(tg, dwx, eye_x);
                const float wy = __builtin_fmaf(tg, dwy, eye_y);
                const float ux = sc.cell_is_one ? wx : wx / sc.cell;
                const float uy = sc.cell_is_one ? wy : wy / sc.cell;
                const int par = ((int)__builtin_floorf(ux) + (int)__builtin_floorf(uy)) & 1;
                c[0] = c[1] = c[2] = par ? sc.gs[1] : sc.gs[0];
            } else {
                const uint32_t g = 0xFFFFFFFFu - low;
                const float4 ns = reinterpret_cast<const float4*>(sc.tri_shade)[g];
                const float* o = body + (sc.tri_idx[g * 2 + 1] >> 16) * kBodyStride;
                float I = __builtin_fmaf(ns.x, o[12], __builtin_fmaf(ns.y, o[13], ns.z * o[14]));
                I = I > 0.0f ? I : 0.0f;
                const float sh = __builtin_fmaf(sc.diffuse, I, sc.ambient);
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    const float v = (o[20 + ch] * ns.w) * sh;
                    c[ch] = v < 1.0f ? v : 1.0f;
                }
            }
            if (mode == PXR_DISTRACT_COLOR) {
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    float v = __builtin_fmaf(c[ch], scale[ch], offs[ch]);
                    v = v > 0.0f ? v : 0.0f;
                    c[ch] = v < 1.0f ? v : 1.0f;
                }
            } else if (mode == PXR_DISTRACT_VIDEO && low <= 1u) {
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    uint32_t byte;
                    if (PX == 4) {
                        const int bi = k * 3 + ch;
                        byte = (vid[bi >> 2] >> ((bi & 3) * 8)) & 0xFFu;
                    } else {
                        byte = vframe[(size_t)p * 3 + ch];
                    }
                    const float vf = (float)byte * (1.0f / 255.0f);
                    c[ch] = __builtin_fmaf(dc.alpha, vf - c[ch], c[ch]);
                }
            }
#pragma unroll
            for (int ch = 0; ch < 3; ++ch) {
                const uint32_t u8 = (uint32_t)(int)__builtin_floorf(__builtin_fmaf(c[ch], 255.0f, 0.5f)) & 0xFFu;
                if (PX == 4) {
                    const int bi = k * 3 + ch;
                    packed[bi >> 2] |= u8 << ((bi & 3) * 8);
                } else {
                    out[(size_t)p * 3 + ch] = (uint8_t)u8;
                }
            }
            idv[k] = 0xFFFFFFFFu - low;
            if (++i == sc.W) {
                i = 0;
                ++j;
            }
        }
        if (PX == 4) {
            uint32_t* dst = reinterpret_cast<uint32_t*>(out) + q * 3;
            struct alignas(4) U3 {
                uint32_t a, b, c;
            };
            *reinterpret_cast<U3*>(dst) = U3{packed[0], packed[1], packed[2]};
            if (out_ids) reinterpret_cast<uint4*>(out_ids)[q] = make_uint4(idv[0], idv[1], idv[2], idv[3]);
        } else {
            if (out_ids) out_ids[p0] = idv[0];
        }
    }
}

template <int NT, int PX>
int launch_one(const SceneConsts& sc, const DistractConsts& dc, const float* d_poses, const float* d_shapes,
               uint32_t n_frames, uint32_t S, uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids,
               hipStream_t stream, std::string& err) {
    hipLaunchKernelGGL((render_kernel<NT, PX>), dim3(n_frames), dim3(NT), sc.lds_total, stream, sc, dc, d_poses, d_shapes, S,
                       step0, env0, d_frames, d_ids);
    const hipError_t rc = hipGetLastError();
    if (rc != hipSuccess) {
        err = std::string("kernel launch failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

template <int NT, int PX>
int prepare_one(uint32_t lds_bytes, std::string& err) {
    const hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&render_kernel<NT, PX>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (rc != hipSuccess) {
        err = std::string("hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

}  // namespace

int prepare_kernels(uint32_t lds_bytes, std::string& err) {
    // The attribute is a per-kernel cap, not a per-launch size: always raise it
    // to the whole 160 KB so that scenes of different sizes can coexist.
    (void)lds_bytes;
    const uint32_t cap = 160u * 1024u;
    int rc;
    if ((rc = prepare_one<256, 4>(cap, err))) return rc;
    if ((rc = prepare_one<512, 4>(cap, err))) return rc;
    if ((rc = prepare_one<1024, 4>(cap, err))) return rc;
    if ((rc = prepare_one<256, 1>(cap, err))) return rc;
    if ((rc = prepare_one<512, 1>(cap, err))) return rc;
    if ((rc = prepare_one<1024, 1>(cap, err))) return rc;
    return PXR_OK;
}

int launch_render(const SceneConsts& sc, const DistractConsts& dc, const float* d_poses, const float* d_shapes,
                  uint32_t n_frames, uint32_t S, uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids,
                  uint32_t block_threads, void* stream, std::string& err) {
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // four pixels per lane need whole 12-byte groups and dword-aligned frames
    const bool quad = (sc.npix % 4u) == 0u;
#define PXR_LAUNCH(NT)                                                                                                   \
    return quad ? launch_one<NT, 4>(sc, dc, d_poses, d_shapes, n_frames, S, step0, env0, d_frames, d_ids, st, err)       \
                : launch_one<NT, 1>(sc, dc, d_poses, d_shapes, n_frames, S, step0, env0, d_frames, d_ids, st, err)
    switch (block_threads) {
        case 256: PXR_LAUNCH(256);
        case 512: PXR_LAUNCH(512);
        case 1024: PXR_LAUNCH(1024);
        default:
            err = "block_threads must be 256, 512 or 1024";
            return PXR_ERR_INVALID_ARG;
    }
#undef PXR_LAUNCH
}

}  // namespace pxr
