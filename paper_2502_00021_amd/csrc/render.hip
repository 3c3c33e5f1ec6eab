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
//   0  per-body transforms, per-frame draws and the three non-triangle colours
//   1  instancing: template vertex -> view space -> snapped fixed point, plus
//      a per-vertex "cell code" saying between which pixel centres it lies
//   2a binning, coarse: one lane per PAIR of edge-sharing triangles; from the
//      cell codes alone (xor / or, no coordinates) decide per triangle whether
//      its bounding box can hold a pixel centre; candidates are compacted
//      wave-wide (ballot + mbcnt) into a list in LDS
//   2b binning, exact: one lane per candidate: exact area sign, pixel range,
//      then compaction into three bins by candidate-pixel count
//   3  raster: bins are walked by 1, 4 or 64 lanes per triangle (rows are
//      dealt round-robin to a triangle's lanes); integer edge functions,
//      top-left rule, float reversed depth, 64-bit LDS atomic max on
//      (depth bits << 32 | ~triangle id)
//   4  resolve: ground ray, id -> flat Lambert colour, distractor, uint8 pack,
//      coalesced 12-byte stores
//
// Floating point is written with explicit fmaf and compiled with
// -ffp-contract=off: the order of operations is part of the output contract
// (coverage is decided by integers derived from these floats).

#include <hip/hip_runtime.h>

#include "arith.h"
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

// Exact products of coordinate differences: 24-bit multiplies when both
// fixed-point extents of the triangle are below 2^15 (every product < 2^30),
// 64-bit otherwise (coordinates reach 2^22, products 2^46).
template <typename I>
__device__ __forceinline__ I emul(int a, int b);
template <>
__device__ __forceinline__ int emul<int>(int a, int b) {
    return __mul24(a, b);
}
template <>
__device__ __forceinline__ long long emul<long long>(int a, int b) {
    return (long long)a * (long long)b;
}

// Walk rows j0 + r, j0 + r + 2^shift, ... of a triangle's candidate pixel range, and in each of them the columns
// i0 + c, i0 + c + 2^cshift, ... (a team of 2^shift x 2^cshift lanes shares the triangle; c = cshift = 0: whole rows).
// Edge functions carry their fill-rule bias and are stepped incrementally; a
// pixel centre is covered when all three are >= 0.
template <typename I>
__device__ __forceinline__ void raster_rows(const TriSetup& s, uint32_t tri, uint32_t W, u64* keys, int r, int shift,
                                            int row_lo, int c = 0, int cshift = 0) {
    int j = s.j0 + r;
    if (j > s.j1) return;
    const int dx_ab = s.bx - s.ax, dy_ab = s.by - s.ay;
    const int dx_bc = s.cx - s.bx, dy_bc = s.cy - s.by;
    const int dx_ca = s.ax - s.cx, dy_ca = s.ay - s.cy;
    const I A2 = emul<I>(dx_ab, s.cy - s.ay) - emul<I>(dy_ab, s.cx - s.ax);
    const float invA = recip_in_range((float)A2);  // a front face: 1 <= A2 < 2^47
    const I b_ab = edge_bias(dx_ab, dy_ab), b_bc = edge_bias(dx_bc, dy_bc), b_ca = edge_bias(dx_ca, dy_ca);
    const int px0 = ((s.i0 + c) << 8) + 128, py = (j << 8) + 128;
    I f_ab = emul<I>(dx_ab, py - s.ay) - emul<I>(dy_ab, px0 - s.ax) + b_ab;
    I f_bc = emul<I>(dx_bc, py - s.by) - emul<I>(dy_bc, px0 - s.bx) + b_bc;
    I f_ca = emul<I>(dx_ca, py - s.cy) - emul<I>(dy_ca, px0 - s.cx) + b_ca;
    const I sx_ab = (I)dy_ab << (8 + cshift), sx_bc = (I)dy_bc << (8 + cshift), sx_ca = (I)dy_ca << (8 + cshift);
    const I sy_ab = (I)dx_ab << (8 + shift), sy_bc = (I)dx_bc << (8 + shift), sy_ca = (I)dx_ca << (8 + shift);
    for (;;) {
        I e_ab = f_ab, e_bc = f_bc, e_ca = f_ca;
        uint32_t pix = (uint32_t)(j - row_lo) * W + (uint32_t)(s.i0 + c);  // the key buffer holds rows from row_lo on
        for (int i = s.i0 + c; i <= s.i1; i += 1 << cshift, pix += 1u << cshift) {
            if ((e_ab | e_bc | e_ca) >= 0) {
                const float beta = (float)(e_ca - b_ca) * invA, gamma = (float)(e_ab - b_ab) * invA;
                z_test(keys, pix, __builtin_fmaf(beta, s.dDb, __builtin_fmaf(gamma, s.dDc, s.Da)), tri);
            }
            e_ab -= sx_ab;
            e_bc -= sx_bc;
            e_ca -= sx_ca;
        }
        j += 1 << shift;
        if (j > s.j1) break;  // (stepping past the last row could leave the exactly representable range)
        f_ab += sy_ab;
        f_bc += sy_bc;
        f_ca += sy_ca;
    }
}

// How a whole wavefront shares a triangle of n rows: 2^shift lanes down the rows (as many as there are rows, up to
// 64), the other 2^(6 - shift) across each row, so that a wide triangle of a few rows (every large triangle of a
// frame that is rendered in bands of a few rows) keeps all lanes busy.
__device__ __forceinline__ void wave_team(int n_rows, int lane, int& r, int& shift, int& c, int& cshift) {
    shift = n_rows >= 33 ? 6 : (32 - __builtin_clz((uint32_t)max(n_rows, 1) * 2u - 1u)) - 1;  // ceil(log2(n_rows))
    cshift = 6 - shift;
    r = lane & ((1 << shift) - 1);
    c = lane >> shift;
}

// Gather the snapped vertices of a triangle (ti = its entry of the index table) and its clamped pixel-centre range.
// Returns kTriNone if a vertex is unusable, all of them lie behind the near plane or no pixel centre is
// inside the bounding box; kTriClip if the triangle straddles the near plane (nothing else is valid
// then); kTriPlain otherwise.  `small_extent` = both fixed-point extents below 2^15.
enum { kTriNone = 0, kTriPlain = 1, kTriClip = 2 };
__device__ __forceinline__ int tri_gather(const SceneConsts& sc, const uint2 ti, const int2* vxy, TriSetup& s,
                                          uint32_t& v0, uint32_t& v1, uint32_t& v2, bool& small_extent) {
    v0 = ti.x & 0xFFFFu;
    v1 = ti.x >> 16;
    v2 = ti.y & 0xFFFFu;
    // (x, y) pairs: one 8-byte LDS read per vertex (as one integer each: read as pairs, the compiler would fetch
    // the y's separately, after the test of the x's, in a second round trip)
    const u64 a = reinterpret_cast<const u64*>(vxy)[v0], b = reinterpret_cast<const u64*>(vxy)[v2], c = reinterpret_cast<const u64*>(vxy)[v1];
    s.ax = (int)(uint32_t)a;
    s.bx = (int)(uint32_t)b;
    s.cx = (int)(uint32_t)c;
    const int minx = imin3(s.ax, s.bx, s.cx), maxx = imax3(s.ax, s.bx, s.cx);
    if (minx <= kBehindX) {  // a sentinel among the three (rare)
        if (minx == kRejectedX) return kTriNone;
        return maxx == kBehindX ? kTriNone : kTriClip;
    }
    s.ay = (int)(uint32_t)(a >> 32);
    s.by = (int)(uint32_t)(b >> 32);
    s.cy = (int)(uint32_t)(c >> 32);
    const int miny = imin3(s.ay, s.by, s.cy), maxy = imax3(s.ay, s.by, s.cy);
    // pixel centres sit at 256 i + 128: first centre >= min, last centre <= max
    s.i0 = max(0, (minx + 127) >> 8);
    s.i1 = min((int)sc.W - 1, (maxx - 128) >> 8);
    s.j0 = max(0, (miny + 127) >> 8);
    s.j1 = min((int)sc.H - 1, (maxy - 128) >> 8);
    small_extent = ((maxx - minx) | (maxy - miny)) < 32768;
    return (s.i0 <= s.i1 && s.j0 <= s.j1) ? kTriPlain : kTriNone;
}

// Which image rows a binned triangle can touch: kTriPlain with [j0, j1] (clamped to the image), or kTriClip for a
// triangle that straddles the near plane (its snapped corners say nothing: it counts for every row).
__device__ __forceinline__ int tri_rows(const SceneConsts& sc, const uint2 ti, const int2* vxy, int& j0, int& j1) {
    const u64 a = reinterpret_cast<const u64*>(vxy)[ti.x & 0xFFFFu], b = reinterpret_cast<const u64*>(vxy)[ti.y & 0xFFFFu],
              c = reinterpret_cast<const u64*>(vxy)[ti.x >> 16];
    if (imin3((int)(uint32_t)a, (int)(uint32_t)b, (int)(uint32_t)c) <= kBehindX) return kTriClip;
    const int ay = (int)(uint32_t)(a >> 32), by = (int)(uint32_t)(b >> 32), cy = (int)(uint32_t)(c >> 32);
    j0 = max(0, (imin3(ay, by, cy) + 127) >> 8);
    j1 = min((int)sc.H - 1, (imax3(ay, by, cy) - 128) >> 8);
    return kTriPlain;
}

// View-space position of template vertex v (the instancing arithmetic of phase 1; also used when a
// triangle has to be clipped).  The template's fourth word says where in LDS its body's record is.
__device__ __forceinline__ void view_position(const SceneConsts& sc, uint32_t v, float& pvx, float& pvy, float& pvz) {
    const float4 tv = reinterpret_cast<const float4*>(sc.vtmpl)[v];
    const uint32_t code = __float_as_uint(tv.w);
    // (body records are 96 bytes at a 16-byte aligned base: four 16-byte LDS reads)
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const __attribute__((address_space(3))) f32x4* o4 =
        reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(static_cast<uintptr_t>(code >> 2));
    const f32x4 m0 = o4[0], m1 = o4[1], m2 = o4[2], sh = o4[4];  // M and t as floats 0..11, the shape as 16..19
    const float sel = (float)(int)__builtin_amdgcn_sbfe((int)code, 0, 2);  // -1, 0 or +1
    const float lx = sh.x * tv.x;
    const float ly = sh.y * tv.y;
    const float lz = __builtin_fmaf(sh.z, tv.z, sel * sh.w);
    pvx = __builtin_fmaf(m0.x, lx, __builtin_fmaf(m0.y, ly, __builtin_fmaf(m0.z, lz, m2.y)));
    pvy = __builtin_fmaf(m0.w, lx, __builtin_fmaf(m1.x, ly, __builtin_fmaf(m1.y, lz, m2.z)));
    pvz = __builtin_fmaf(m1.z, lx, __builtin_fmaf(m1.w, ly, __builtin_fmaf(m2.x, lz, m2.w)));
}

// One piece (a, b, c in screen order) of a clipped triangle, rastered by a whole wavefront.
__device__ __forceinline__ void raster_piece(const SceneConsts& sc, uint32_t t, int ax, int ay, float Da, int bx, int by,
                                             float Db, int cx, int cy, float Dc, bool usable, u64* keys, int lane,
                                             int row_lo, int row_hi) {
    if (!usable) return;
    if (!((long long)(bx - ax) * (long long)(cy - ay) > (long long)(by - ay) * (long long)(cx - ax))) return;  // back face
    TriSetup s;
    s.ax = ax; s.ay = ay; s.bx = bx; s.by = by; s.cx = cx; s.cy = cy;
    const int minx = imin3(ax, bx, cx), maxx = imax3(ax, bx, cx), miny = imin3(ay, by, cy), maxy = imax3(ay, by, cy);
    s.i0 = max(0, (minx + 127) >> 8);
    s.i1 = min((int)sc.W - 1, (maxx - 128) >> 8);
    s.j0 = max(max(0, (miny + 127) >> 8), row_lo);
    s.j1 = min(min((int)sc.H - 1, (maxy - 128) >> 8), row_hi - 1);
    if (s.i0 > s.i1 || s.j0 > s.j1) return;
    s.Da = Da;
    s.dDb = Db - Da;
    s.dDc = Dc - Da;
    int r, shift, c, cshift;
    wave_team(s.j1 - s.j0 + 1, lane, r, shift, c, cshift);
    if (((maxx - minx) | (maxy - miny)) < 32768)
        raster_rows<int>(s, t, sc.W, keys, r, shift, row_lo, c, cshift);
    else
        raster_rows<long long>(s, t, sc.W, keys, r, shift, row_lo, c, cshift);
}

// A triangle with corners on both sides of the near plane (every lane of the wavefront computes the
// same clip).  Walk the edges v0->v1, v1->v2, v2->v0: a corner in front is kept, an edge that crosses
// the plane adds its intersection, computed from the corner in front (P) towards the one behind (Q) so
// that both triangles sharing the edge get the same point:
//   t = (z_near - P.z) / (Q.z - P.z),  I = (fma(t, Q.x - P.x, P.x), fma(t, Q.y - P.y, P.y), z_near).
// The 3 or 4 corners w0.. keep the winding; new ones are projected and snapped like template vertices
// (outside the guard band = unusable) and the pieces (w0,w1,w2), (w0,w2,w3) are rastered under id t.
//
// Which corner the walk emits k-th depends only on which of the three vertices are in front: a 4-bit
// code per corner (P << 2 | Q, P == Q for a kept vertex), four corners per pattern, patterns indexed by
// the in-front mask (bit e = vertex e in front).  Corners are recomputed per piece rather than kept, so
// that this rarely taken path does not raise the kernel's register count.
__device__ __forceinline__ void raster_clipped(const SceneConsts& sc, uint32_t t, const int2* vxy,
                                               const float* vd, u64* keys, int lane, int row_lo, int row_hi) {
#pragma unroll 1
    for (uint32_t piece = 0; piece < 2u; ++piece) {
        // everything is re-derived per piece so that nothing but `t` stays live across the raster loops
        const uint2 ti = reinterpret_cast<const uint2*>(sc.tri_idx)[t];
        const uint32_t v0 = ti.x & 0xFFFFu, v1 = ti.x >> 16, v2 = ti.y & 0xFFFFu;
        const uint32_t mask = (vxy[v0].x != kBehindX ? 1u : 0u) | (vxy[v1].x != kBehindX ? 2u : 0u) | (vxy[v2].x != kBehindX ? 4u : 0u);
        // corners k = 0..3 in bits 4k..4k+3; V_e = e<<2|e, I_pq = p<<2|q
        //   001: V0 I01 I02      010: I10 V1 I12      100: I21 V2 I20
        //   011: V0 V1 I12 I02   110: I10 V1 V2 I20   101: V0 I01 I21 V2
        const uint32_t pattern = mask == 1u ? 0x0210u : mask == 2u ? 0x0654u : mask == 4u ? 0x08A9u
                               : mask == 3u ? 0x2650u : mask == 6u ? 0x8A54u : 0xA910u;
        if (piece == 1u && (mask == 1u || mask == 2u || mask == 4u)) break;  // one corner in front: one piece
        const float inv = 1.0f / sc.z_near;
        // screen order (a, b, c) = (w0, w2, w1), then (w0, w3, w2)
        const uint32_t order = piece == 0 ? 0x120u : 0x230u;
        int cX[3], cY[3];
        float cD[3];
        bool usable = true;
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const uint32_t code = (pattern >> (4u * ((order >> (4 * c)) & 15u))) & 15u;
            const uint32_t p = code >> 2, q = code & 3u;
            const uint32_t vp = p == 0 ? v0 : (p == 1 ? v1 : v2), vq = q == 0 ? v0 : (q == 1 ? v1 : v2);
            if (p == q) {
                cX[c] = vxy[vp].x;
                cY[c] = vxy[vp].y;
                cD[c] = vd[vp];
            } else {
                float px, py, pz, qx, qy, qz;
                view_position(sc, vp, px, py, pz);
                __builtin_amdgcn_sched_barrier(0);  // one vertex at a time: keeps this path within the register budget
                view_position(sc, vq, qx, qy, qz);
                __builtin_amdgcn_sched_barrier(0);
                const float tt = (sc.z_near - pz) / (qz - pz);
                const float ix = __builtin_fmaf(tt, qx - px, px);
                const float iy = __builtin_fmaf(tt, qy - py, py);
                const float sx = __builtin_fmaf(sc.f, ix * inv, sc.halfW);
                const float sy = __builtin_fmaf(-sc.f, iy * inv, sc.halfH);
                const bool ok = (__builtin_fabsf(sx) <= 16384.0f) && (__builtin_fabsf(sy) <= 16384.0f);
                usable = usable && ok;
                cX[c] = ok ? floor_to_int(__builtin_fmaf(sx, 256.0f, 0.5f)) : 0;
                cY[c] = ok ? floor_to_int(__builtin_fmaf(sy, 256.0f, 0.5f)) : 0;
                cD[c] = sc.z_near * inv;
            }
        }
        raster_piece(sc, t, cX[0], cY[0], cD[0], cX[1], cY[1], cD[1], cX[2], cY[2], cD[2], usable, keys, lane, row_lo, row_hi);
    }
}

// Raster one binned triangle with lane `r` of the 2^shift lanes that share it, restricted to
// the rows [row_lo, row_hi) that the key buffer currently holds.
// MAY_CLIP: the bin (the wave-per-triangle one) also holds the triangles that straddle the near plane.
template <bool MAY_CLIP>
__device__ __forceinline__ void raster_binned(const SceneConsts& sc, uint32_t t, const uint2 ti,
                                              const int2* vxy, const float* vd, u64* keys, int r, int shift, int row_lo,
                                              int row_hi) {
    TriSetup s;
    uint32_t v0, v1, v2;
    bool small_extent;
    const int kind = tri_gather(sc, ti, vxy, s, v0, v1, v2, small_extent);
    if (MAY_CLIP && kind == kTriClip) {
        raster_clipped(sc, t, vxy, vd, keys, r, row_lo, row_hi);
        return;
    }
    s.j0 = max(s.j0, row_lo);
    s.j1 = min(s.j1, row_hi - 1);
    if (s.j0 > s.j1) return;
    s.Da = vd[v0];
    s.dDb = vd[v2] - s.Da;
    s.dDc = vd[v1] - s.Da;
    int c = 0, cshift = 0;
    if (MAY_CLIP) wave_team(s.j1 - s.j0 + 1, r, r, shift, c, cshift);  // (the wave-per-triangle bin: r is the lane)
    if (small_extent)
        raster_rows<int>(s, t, sc.W, keys, r, shift, row_lo, c, cshift);
    else
        raster_rows<long long>(s, t, sc.W, keys, r, shift, row_lo, c, cshift);
}

// Per-axis cell code of a snapped coordinate for an image of n pixels:
// 2g = strictly between pixel centres g-1 and g, 2c+1 = exactly on centre c,
// clamped to [0, 2n] (0 = left of centre 0, 2n = right of centre n-1).  A set
// of points has no pixel centre within its extent along this axis iff all
// codes are equal and even.
__device__ __forceinline__ uint32_t cell_code(int x, int n) {
    const int f = ((x - 128) >> 8) + ((x + 127) >> 8) + 1;
    int r;
    asm("v_med3_i32 %0, %1, 0, %2" : "=v"(r) : "v"(f), "s"(2 * n));  // clamp(f, 0, 2n) in one instruction (n > 0)
    return (uint32_t)r;
}

// A 32-bit word of LDS by its byte address.  (The dynamic LDS segment starts at address 0: the kernels here have
// no static LDS, which prepare_kernels verifies; tables built on the host can therefore hold LDS addresses.)
__device__ __forceinline__ uint32_t lds_u32_at(uint32_t byte_address) {
    return *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(static_cast<uintptr_t>(byte_address));
}

// Low half times high half of a word (non-zero iff both are), in one instruction.
__device__ __forceinline__ uint32_t halves_product(uint32_t x) {
    uint32_t r;
    asm("v_mul_u32_u24_sdwa %0, %1, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:WORD_0" : "=v"(r) : "v"(x));
    return r;
}

__device__ __forceinline__ uint32_t lanes_below(u64 m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t quantise(float c) {
    return (uint32_t)floor_to_int(__builtin_fmaf(c, 255.0f, 0.5f)) & 0xFFu;
}

// ---------------------------------------------------------------- the kernel

// The kernel's first two (by-value) arguments, read afresh from the kernel-argument segment: whatever the
// compiler loaded from them before is not reused after this point.  The band loop of tall frames takes its
// constants through this at the top of every trip, so that they are fetched again (scalar loads that hit the
// constant cache) instead of being kept in scalar registers across the whole loop, which the 1024-thread
// variants do not have.
constexpr uint32_t kSceneArgAt = 0;
constexpr uint32_t kDistractArgAt = (sizeof(SceneConsts) + alignof(DistractConsts) - 1) / alignof(DistractConsts) * alignof(DistractConsts);
template <typename T>
__device__ __forceinline__ const T& argument_reloaded(uint32_t byte_offset) {
    typedef const __attribute__((address_space(4))) unsigned char* KernargBytes;
    KernargBytes p = (KernargBytes)__builtin_amdgcn_kernarg_segment_ptr() + byte_offset;
    asm volatile("" : "+s"(p));
    return *(const T*)(const __attribute__((address_space(4))) T*)p;
}

// Phase probes: empty in the library.  A profiling build (-DPXR_PROFILING_BUILD, made into a file of its own
// by build.py --define) takes them from a header that the library's build never includes.
#ifdef PXR_PROFILING_BUILD
#include "profiling/phase_probes.h"
#else
#define PXR_PHASE_BEGIN()
#define PXR_PHASE_MARK(i)
#define PXR_TIMED_BARRIER(i) __syncthreads()
#define PXR_PHASE_END()
#endif

struct FrameUniforms {  // written in phase 0 (one lane) or by LDS atomics, read by all after a barrier
    u64 bins;           // three 16-bit counters: tiny | small << 16 | large << 32
    uint32_t n_cand;
    uint32_t video_frame;
    float scale[3], offs[3];
    float base_col[3][3];     // background, ground grey 0, ground grey 1 after the colour distractor
    uint32_t base_packed[3];  // the same three, quantised: R | G<<8 | B<<16
    float eye[3];             // camera position (written by the first lane in phase 0 for phase 4)
    uint32_t pad_;
    u64 band_bins[2];         // banded frames: the three counters of one band round's lists, double-buffered by round
};

// Everything phase 4 needs that is uniform over the frame.
static_assert((offsetof(FrameUniforms, base_packed) + 4) % 8 == 0, "the first grey's word must be 8-byte aligned");

struct ResolveCtx {
    float eye_x, eye_y, eye_z, inv_ez;
    bool ground_ok;
    uint32_t mode;
    float alpha;
    float scale[3], offs[3];
    uint32_t col_addr;     // LDS byte address of the three colours as floats [3][3]
    uint32_t packed_addr;  // and as packed bytes [3]
    uint32_t vlut;         // LDS byte address of the video-blend tables, 0 = none
    const uint8_t* vframe;
};

// Ground plane z = 0 along the pixel's ray: returns its z-test key (0 = miss)
// and the ray parameter (= view depth) of the hit.
__device__ __forceinline__ u64 ground_key(const SceneConsts& sc, const ResolveCtx& rc, float ndz, float& tg) {
    tg = 0.0f;
    if (rc.ground_ok && ndz > 0.0f) {
        tg = rc.eye_z / ndz;
        if (tg >= sc.z_near && tg <= sc.z_far) {
            const float dg = (sc.z_near * ndz) * rc.inv_ez;
            return ((u64)__float_as_uint(dg) << 32) | 1ull;
        }
    }
    return 0ull;
}

// One pixel: winner of (triangles, ground, background) -> colour -> distractor
// -> 24-bit RGB.  `low` returns ~id.  `vbytes` = the pixel's three video bytes
// (R | G<<8 | B<<16), only read in video mode.
// UNIT_CELL: the checkerboard cell is 1 m, so the division by the cell size is the identity, and the ground point
// cannot be a NaN (a finite or infinite eye, a far plane within 2^64), so the one-instruction floor-and-convert serves.
// Triangle g as a 24-bit colour: flat Lambert + ambient in the body frame, then the colour distractor.
template <bool VIDEO>
__device__ __forceinline__ uint32_t shade_triangle(const SceneConsts& sc, const ResolveCtx& rc, const float* body, uint32_t g) {
    const float4 ns = reinterpret_cast<const float4*>(sc.tri_shade)[g];
    const float4* o4 = reinterpret_cast<const float4*>(body + (sc.tri_idx[g * 2 + 1] >> 16) * kBodyStride);
    const float4 lb = o4[3], col = o4[5];  // floats 12..14: light in the body frame, 20..22: colour
    const float o_rgb[3] = {col.x, col.y, col.z};
    float I = __builtin_fmaf(ns.x, lb.x, __builtin_fmaf(ns.y, lb.y, ns.z * lb.z));
    I = I > 0.0f ? I : 0.0f;
    const float sh = __builtin_fmaf(sc.diffuse, I, sc.ambient);
    uint32_t rgb = 0;
#pragma unroll
    for (int ch = 0; ch < 3; ++ch) {
        float v = (o_rgb[ch] * ns.w) * sh;
        v = v < 1.0f ? v : 1.0f;
        if (!VIDEO && rc.mode == PXR_DISTRACT_COLOR) {
            v = __builtin_fmaf(v, rc.scale[ch], rc.offs[ch]);
            v = v > 0.0f ? v : 0.0f;
            v = v < 1.0f ? v : 1.0f;
        }
        rgb |= quantise(v) << (8 * ch);
    }
    return rgb;
}

// Sum of the two checker cell indices where the pixel's ray (parameter tg, direction dwx, dwy) meets the ground:
// its lowest bit says which of the two greys shows.
template <bool UNIT_CELL>
__device__ __forceinline__ uint32_t checker_cells(const SceneConsts& sc, const ResolveCtx& rc, float tg, float dwx, float dwy) {
    const float wx = __builtin_fmaf(tg, dwx, rc.eye_x);
    const float wy = __builtin_fmaf(tg, dwy, rc.eye_y);
    if (UNIT_CELL)  // (wx and wy are no NaNs here: the caller has looked at the eye and at z_far)
        return (uint32_t)floor_to_int(wx) + (uint32_t)floor_to_int(wy);
    return (uint32_t)(int)__builtin_floorf(wx / sc.cell) + (uint32_t)(int)__builtin_floorf(wy / sc.cell);
}

// DEFER_TRIANGLES: a triangle pixel returns 0 here; the caller shades it (compacted over the wavefront).
template <bool UNIT_CELL, bool VIDEO, bool DEFER_TRIANGLES = false>
__device__ __forceinline__ uint32_t resolve_pixel(const SceneConsts& sc, const ResolveCtx& rc, const float* body, u64 key,
                                                  u64 gkey, float tg, float dwx, float dwy, uint32_t vbytes, uint32_t& low,
                                                  u64& tri_lanes) {
    key = key > gkey ? key : gkey;
    low = (uint32_t)key;
    tri_lanes = __ballot(low > 1u);  // (taken here, beside the branch on the same comparison, it costs nothing)
    if (low > 1u) return DEFER_TRIANGLES ? 0u : shade_triangle<VIDEO>(sc, rc, body, 0xFFFFFFFFu - low);
    // background or ground: one of three colours per frame (consecutive in LDS: background, grey 0, grey 1)
    if (!VIDEO) {
        uint32_t word = rc.packed_addr;
        if (low == 1u) word = rc.packed_addr + 4u + ((checker_cells<UNIT_CELL>(sc, rc, tg, dwx, dwy) & 1u) << 2);
        return lds_u32_at(word);
    }
    uint32_t col = rc.col_addr;
    if (low == 1u) {
        uint32_t grey = checker_cells<UNIT_CELL>(sc, rc, tg, dwx, dwy) & 1u;
        asm("" : "+v"(grey));  // (kept from the compiler, which would turn the multiply-add into compare, select, add)
        col = __umul24(grey, 12u) + (rc.col_addr + 12u);
    }
    const __attribute__((address_space(3))) float* c3 =
        reinterpret_cast<const __attribute__((address_space(3))) float*>(static_cast<uintptr_t>(col));
    uint32_t rgb = 0;
#pragma unroll
    for (int ch = 0; ch < 3; ++ch) {
        const float c = c3[ch];
        const float vf = (float)((vbytes >> (8 * ch)) & 0xFFu) * (1.0f / 255.0f);
        rgb |= quantise(__builtin_fmaf(rc.alpha, vf - c, c)) << (8 * ch);
    }
    return rgb;
}

// Phase 4 for images whose width is a multiple of 4: four consecutive pixels of one row per
// lane.  The row part of the ray is shared, and without camera roll (NO_ROLL: the right vector is
// horizontal) so is the whole ground test, which then costs one division per lane, not four.
template <int NT, bool UNIT_CELL, bool NO_ROLL, bool VIDEO, bool SELF_CLEAR>
__device__ __forceinline__ void resolve_rows4(const SceneConsts& sc, const ResolveCtx& rc, const float* body,
                                              const float* cxcy, const float4* rows, u64* keys, uint8_t* out,
                                              uint32_t* out_ids, uint32_t tid, uint32_t p_begin, uint32_t p_end) {
    // pixels [p_begin, p_end) of the frame; keys[0] belongs to pixel p_begin
    const uint32_t lane = tid & 63u;
    for (uint32_t q = (p_begin >> 2) + tid; q * 4 < p_end; q += NT) {
        const uint32_t p0 = q * 4;
        const uint32_t j = __umulhi(p0, sc.magicW);
        const uint32_t i0 = p0 - j * sc.W;
        // what is shared by a row's pixels was worked out once per row in phase 0
        const float4 row = rows[j];
        const float rx = row.x, ry = row.y;
        const float rz = NO_ROLL ? 0.0f : row.z;
        const float4 cx4 = *reinterpret_cast<const float4*>(cxcy + i0);
        const float cxs[4] = {cx4.x, cx4.y, cx4.z, cx4.w};
        uint32_t vid[3] = {0u, 0u, 0u};
        if (VIDEO) {
            const uint32_t* vsrc = reinterpret_cast<const uint32_t*>(rc.vframe) + q * 3;
            vid[0] = vsrc[0];
            vid[1] = vsrc[1];
            vid[2] = vsrc[2];
        }
        const uint32_t vb[4] = {vid[0] & 0xFFFFFFu, (vid[0] >> 24) | ((vid[1] & 0xFFFFu) << 8),
                                (vid[1] >> 16) | ((vid[2] & 0xFFu) << 16), vid[2] >> 8};
        // without roll the ground test is the row's: ray parameter (0 = miss) and depth bits from the row table
        const float tg_row = NO_ROLL ? row.z : 0.0f;
        // (a miss has depth bits 0 in the table: the key is 0 then)
        const u64 gkey_row = NO_ROLL ? (((u64)__float_as_uint(row.w) << 32) | (tg_row != 0.0f ? 1ull : 0ull)) : 0ull;
        // the lane's four keys are 32 contiguous, aligned bytes: two 16-byte LDS reads
        const uint4 k01 = reinterpret_cast<const uint4*>(keys + (p0 - p_begin))[0], k23 = reinterpret_cast<const uint4*>(keys + (p0 - p_begin))[1];
        const u64 key4[4] = {((u64)k01.y << 32) | k01.x, ((u64)k01.w << 32) | k01.z, ((u64)k23.y << 32) | k23.x, ((u64)k23.w << 32) | k23.z};
        uint32_t rgb[4] = {0u, 0u, 0u, 0u}, low[4];
        uint32_t ow[3] = {0u, 0u, 0u};  // the 12 bytes that leave
        bool direct = false;            // they were put together as they were looked up (rgb[] is not used)
        u64 tri_lanes[4];
        if (!VIDEO) {
            // One of the frame's three colours (background, two greys: consecutive words in LDS), without a branch
            // per pixel.  A triangle pixel picks up one of them as well, to be overwritten below.  Without roll a
            // row is ground or sky as a whole, so the choice between "background" and "a grey by the checker" is the
            // lane's, not the pixel's.
            const bool ground_row = tg_row != 0.0f;
            // (the first grey sits at a multiple of 8 bytes: "+ 4 for the second" is an "or")
            const uint32_t lane_word = rc.packed_addr + ((NO_ROLL && ground_row) ? 4u : 0u);
            const uint32_t lane_mask = (NO_ROLL && ground_row) ? 4u : 0u;
            const bool ground_in_sight = !NO_ROLL || __ballot(ground_row) != 0ull;  // (a wavefront above the horizon)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float tg = tg_row;
                u64 gkey = gkey_row;
                if (!NO_ROLL) gkey = ground_key(sc, rc, -__builtin_fmaf(sc.Rt[2], cxs[k], rz), tg);
                const u64 key = key4[k] > gkey ? key4[k] : gkey;
                low[k] = (uint32_t)key;
                tri_lanes[k] = __ballot(low[k] > 1u);
                uint32_t word = lane_word;
                if (ground_in_sight) {
                    const float dwx = __builtin_fmaf(sc.Rt[0], cxs[k], rx);
                    const float dwy = __builtin_fmaf(sc.Rt[1], cxs[k], ry);
                    const uint32_t cells = checker_cells<UNIT_CELL>(sc, rc, tg, dwx, dwy);
                    if (NO_ROLL)
                        word = lane_word | ((cells << 2) & lane_mask);
                    else
                        word = low[k] == 1u ? rc.packed_addr + 4u + ((cells & 1u) << 2) : rc.packed_addr;
                }
                rgb[k] = lds_u32_at(word);
            }
        } else if (NO_ROLL && rc.vlut) {
            // Video distractor, no roll, tables in LDS: a row is sky or ground as a whole, so under the clip lies
            // the background or one of the two greys by the checker's parity, and the blended byte of a channel
            // is one byte read from the table of that colour, indexed by the clip's byte where it lies in the three
            // words that brought it (byte n = channel n % 3 of pixel n / 3), and put at the same place of the three
            // words that leave.  A triangle pixel gets a blended colour as well, replaced below.
            direct = true;
            const bool ground_row = tg_row != 0.0f;
            const uint32_t lane_base = rc.vlut + (ground_row ? 768u : 0u);  // background's tables, or the first grey's
            const uint32_t odd_step = ground_row ? 768u : 0u;               // the second grey's follow the first's
            uint32_t base[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u64 key = key4[k] > gkey_row ? key4[k] : gkey_row;
                low[k] = (uint32_t)key;
                tri_lanes[k] = __ballot(low[k] > 1u);
                const float dwx = __builtin_fmaf(sc.Rt[0], cxs[k], rx);
                const float dwy = __builtin_fmaf(sc.Rt[1], cxs[k], ry);
                uint32_t odd = checker_cells<UNIT_CELL>(sc, rc, tg_row, dwx, dwy) & 1u;
                asm("" : "+v"(odd));  // (kept from the compiler, which would turn the multiply-add into compare, select, add)
                base[k] = __umul24(odd, odd_step) + lane_base;
            }
#pragma unroll
            for (int w = 0; w < 3; ++w) {
                uint32_t word = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int n = 4 * w + b;
                    const uint32_t at = base[n / 3] + ((vid[w] >> (8 * b)) & 0xFFu) + 256u * (n % 3);
                    word |= (uint32_t)*reinterpret_cast<const __attribute__((address_space(3))) uint8_t*>(static_cast<uintptr_t>(at)) << (8 * b);
                }
                ow[w] = word;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float tg = tg_row;
                u64 gkey = gkey_row;
                if (!NO_ROLL) gkey = ground_key(sc, rc, -__builtin_fmaf(sc.Rt[2], cxs[k], rz), tg);
                const float dwx = __builtin_fmaf(sc.Rt[0], cxs[k], rx);
                const float dwy = __builtin_fmaf(sc.Rt[1], cxs[k], ry);
                rgb[k] = resolve_pixel<UNIT_CELL, VIDEO, true>(sc, rc, body, key4[k], gkey, tg, dwx, dwy, vb[k], low[k], tri_lanes[k]);
            }
        }
        // Triangle pixels are few and clustered: instead of every lane walking the shading code four
        // times, the wavefront compacts its triangle pixels into a list (in the LDS of its own, already
        // consumed, pixel keys), shades the list densely, and the owners pick their colours up.
        const u64 m0 = tri_lanes[0], m1 = tri_lanes[1], m2 = tri_lanes[2], m3 = tri_lanes[3];
        if (m0 | m1 | m2 | m3) {
            uint32_t* list = reinterpret_cast<uint32_t*>(keys + ((q - lane) * 4 - p_begin));  // 256 keys = 512 words
            const uint32_t n0 = (uint32_t)__popcll(m0), n1 = n0 + (uint32_t)__popcll(m1), n2 = n1 + (uint32_t)__popcll(m2);
            const uint32_t total = n2 + (uint32_t)__popcll(m3);
            const uint32_t slot[4] = {lanes_below(m0), n0 + lanes_below(m1), n1 + lanes_below(m2), n2 + lanes_below(m3)};
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (low[k] > 1u) list[slot[k]] = low[k];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const u64 active = __ballot(true);  // the last trip of a ragged band may run with fewer lanes
            for (uint32_t i = lanes_below(active); i < total; i += (uint32_t)__popcll(active))
                list[i] = shade_triangle<VIDEO>(sc, rc, body, 0xFFFFFFFFu - list[i]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (low[k] > 1u) rgb[k] = list[slot[k]];
            if (VIDEO && direct) {
                // (pixel k's three bytes start at byte 3 k of the twelve)
                if (low[0] > 1u) ow[0] = (ow[0] & 0xFF000000u) | rgb[0];
                if (low[1] > 1u) {
                    ow[0] = (ow[0] & 0x00FFFFFFu) | (rgb[1] << 24);
                    ow[1] = (ow[1] & 0xFFFF0000u) | (rgb[1] >> 8);
                }
                if (low[2] > 1u) {
                    ow[1] = (ow[1] & 0x0000FFFFu) | (rgb[2] << 16);
                    ow[2] = (ow[2] & 0xFFFFFF00u) | (rgb[2] >> 16);
                }
                if (low[3] > 1u) ow[2] = (ow[2] & 0x000000FFu) | (rgb[3] << 8);
            }
        }
        if (SELF_CLEAR) {
            // banded frames: the lane leaves its four keys cleared for the next band (nobody else touches them)
            reinterpret_cast<uint4*>(keys + (p0 - p_begin))[0] = make_uint4(0u, 0u, 0u, 0u);
            reinterpret_cast<uint4*>(keys + (p0 - p_begin))[1] = make_uint4(0u, 0u, 0u, 0u);
        }
        if (!(VIDEO && direct)) {
            ow[0] = rgb[0] | (rgb[1] << 24);
            ow[1] = (rgb[1] >> 8) | (rgb[2] << 16);
            ow[2] = (rgb[2] >> 16) | (rgb[3] << 8);
        }
        struct alignas(4) U3 {
            uint32_t a, b, c;
        };
        *reinterpret_cast<U3*>(reinterpret_cast<uint32_t*>(out) + q * 3) = U3{ow[0], ow[1], ow[2]};
        if (out_ids)
            reinterpret_cast<uint4*>(out_ids)[q] =
                make_uint4(0xFFFFFFFFu - low[0], 0xFFFFFFFFu - low[1], 0xFFFFFFFFu - low[2], 0xFFFFFFFFu - low[3]);
    }
}

// Register budget: two 80 KB workgroups share a compute unit, so 1024-thread groups need all
// 8 wave slots per SIMD (<= 64 VGPRs); the smaller groups may use more registers.
// BANDED: the key buffer holds only `band_rows` rows at a time and phases 3-4 loop over bands.
template <int NT, int PX, bool BANDED, bool VIDEO>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(NT >= 1024 ? 8 : (NT >= 768 ? 6 : 4)))) void render_kernel(
    const SceneConsts sc, const DistractConsts dc, const float* __restrict__ poses, const float* __restrict__ shapes,
    uint32_t S, uint32_t step0, uint32_t env0, uint8_t* __restrict__ frames, uint32_t* __restrict__ ids) {
    extern __shared__ __align__(16) unsigned char lds[];
    // the key buffer's LDS holds the cell codes and the candidate list until the keys are cleared
    uint32_t* vm = reinterpret_cast<uint32_t*>(lds + sc.lds_keys);
    uint16_t* cand = reinterpret_cast<uint16_t*>(lds + sc.lds_keys + sc.V * 4 + 4);  // (after the word of code 0)
    int2* vxy = reinterpret_cast<int2*>(lds + sc.lds_vxy);
    float* vd = reinterpret_cast<float*>(lds + sc.lds_vd);
    float* body = reinterpret_cast<float*>(lds + sc.lds_body);
    float* cxcy = reinterpret_cast<float*>(lds + sc.lds_cxcy);
    float4* rows = reinterpret_cast<float4*>(lds + sc.lds_rows);
    FrameUniforms* fu = reinterpret_cast<FrameUniforms*>(lds + sc.lds_misc);
    uint16_t* list = reinterpret_cast<uint16_t*>(lds + sc.lds_list);    // tiny bin grows up, small bin grows down
    uint16_t* list2 = reinterpret_cast<uint16_t*>(lds + sc.lds_large);  // large bin

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t frame = frame_of_block(blockIdx.x, gridDim.x);
    const uint32_t e = frame / S;
    const uint32_t step = step0 + (frame - e * S);
    const uint32_t env = env0 + e;
    const float* pose = poses + (size_t)frame * sc.K * 7;

    // camera position: fixed world-space offset from the root body.
    // The root's position is fetched with vector loads (through an offset of 0 that the compiler cannot see
    // through), although it is the same for every lane: as scalar loads they share their counter with the loads
    // of the kernel's arguments, every wait for one of those would wait for memory as well, and the first
    // wavefront would request its bodies' poses only after the root's position had arrived.
    uint32_t opaque_zero = 0u;
    asm volatile("" : "+v"(opaque_zero));
    const float* root_pos = pose + sc.root * 7 + opaque_zero;
    // (Only requested here.  The additions, and with them the wait, are made where phase 0 uses the eye: after the
    // bodies' lanes have requested their poses, in particular.  Phase 4 gets the eye through LDS, so that these
    // registers are free in between.)
    const float root_x = root_pos[0], root_y = root_pos[1], root_z = root_pos[2];

    PXR_PHASE_BEGIN();
    // ---- phase 0: per-body transforms, per-frame draws, the three non-triangle colours
    // (16-wavefront groups: copied by the fourth wavefront on, the first three have chains of their own in this
    // phase; measured the other way round for the smaller groups)
    constexpr uint32_t kCopyFrom = NT >= 1024 ? 192u : 0u;
    if (tid >= kCopyFrom)
        for (uint32_t i = tid - kCopyFrom; i < sc.W + sc.H; i += NT - kCopyFrom) cxcy[i] = sc.cxcy[i];
    if (tid < 4u * sc.K) {
        // Four lanes per body: each rebuilds the body's rotation and takes one row of the work (the view matrix
        // has three rows, the light direction is the fourth): a quarter of the dot products on the chain.
        const uint32_t b = tid >> 2, part = tid & 3u;
        const float* p = pose + b * 7;
        // Everything the lane will need from memory is requested here, in one go: the pose, the lane's row of
        // (right, up, forward, light) from the table behind the bodies' constants, the body's shape and colour
        // (all four lanes of a body ask for the same: one request).
        const float* vr = sc.body_const + sc.K * 8u + 3u * part;
        const float r0 = vr[0], r1 = vr[1], r2 = vr[2];
        const float4 shp = *reinterpret_cast<const float4*>(shapes ? shapes + ((size_t)e * sc.K + b) * 4 : sc.body_const + b * 8);
        const float4 col = *reinterpret_cast<const float4*>(sc.body_const + b * 8 + 4);
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
        const float eye_x = root_x + sc.off[0], eye_y = root_y + sc.off[1], eye_z = root_z + sc.off[2];
        const float dx = p[0] - eye_x, dy = p[1] - eye_y, dz = p[2] - eye_z;
        if (tid == 0u) {
            fu->eye[0] = eye_x;
            fu->eye[1] = eye_y;
            fu->eye[2] = eye_z;
        }
        float* o = body + b * kBodyStride;
#pragma unroll
        for (int c = 0; c < 3; ++c) o[3u * part + (part == 3u ? 3u : 0u) + c] = dot3(r0, r1, r2, R[0][c], R[1][c], R[2][c]);
        if (part < 3u) o[9u + part] = dot3(r0, r1, r2, dx, dy, dz);
        // (written by all four lanes, the same values: in a branch of its own the compiler would request them
        // only there, after the arithmetic, and the first wavefront would wait for memory twice)
        *reinterpret_cast<float4*>(o + 16) = shp;
        *reinterpret_cast<float4*>(o + 20) = col;  // (the fourth float is padding)
    }
    if (tid >= 64u) {
        // The second wavefront on: one lane per image row prepares what all pixels of the row share: the row
        // part of the ray, and - when the camera does not roll, so that the ray's z does not depend on the
        // column (fma(+-0, cx, rz) == rz) - the whole ground test with its division.
        //   rows[j] = (rx, ry, tg or 0 for a miss, depth bits)   without roll
        //   rows[j] = (rx, ry, rz, -)                            with roll
        const bool no_roll = sc.Rt[2] == 0.0f;
        ResolveCtx g;
        const float eye_z = root_z + sc.off[2];
        g.eye_z = eye_z;
        g.inv_ez = 1.0f / eye_z;
        g.ground_ok = sc.ground_on && eye_z > 0.0f;
        for (uint32_t j = tid - 64u; j < sc.H; j += NT - 64u) {
            const float cyj = sc.cxcy[sc.W + j];
            const float rz = __builtin_fmaf(sc.Up[2], cyj, sc.Fw[2]);
            float4 r;
            r.x = __builtin_fmaf(sc.Up[0], cyj, sc.Fw[0]);
            r.y = __builtin_fmaf(sc.Up[1], cyj, sc.Fw[1]);
            r.z = rz;
            r.w = 0.0f;
            if (no_roll) {
                float tg;
                const u64 key = ground_key(sc, g, -rz, tg);
                r.z = key ? tg : 0.0f;  // (a hit has tg >= z_near > 0)
                r.w = __uint_as_float((uint32_t)(key >> 32));
            }
            rows[j] = r;
        }
    }
    // (The wavefronts of a workgroup start a few hundred clocks apart, four at a time; the last ones start more than
    // a thousand clocks after the first.  The draws are this phase's longest chain beside the bodies': they belong on
    // an early wavefront that has nothing else to do - the third - and the late ones get no work here at all.)
    constexpr uint32_t kDrawLane = NT >= 1024 ? 191u : NT - 1u;  // last lane of the third wavefront (of the last: smaller groups)
    if (!VIDEO && tid <= kDrawLane && tid >= kDrawLane - 1u && dc.mode == PXR_DISTRACT_COLOR) {
        // The colour draws are two generator streams, the longest serial chain of this phase: the two
        // lanes walk one stream each, side by side; the offsets go through LDS to the last lane.
        const uint32_t stream = kDrawLane - tid;
        uint32_t r[4];
        counter_rng(dc.seed_lo, dc.seed_hi, env, step, stream, 0u, r);
        const float span = stream == 0u ? dc.scale_span : dc.offset_span, lo = stream == 0u ? dc.scale_lo : dc.offset_lo;
        float* dst = stream == 0u ? fu->scale : fu->offs;
#pragma unroll
        for (int c = 0; c < 3; ++c) dst[c] = __builtin_fmaf(unit_float(r[c]), span, lo);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (tid == kDrawLane) {
        fu->bins = 0ull;
        fu->n_cand = 0;
        if (BANDED) fu->band_bins[0] = fu->band_bins[1] = 0ull;
        if (VIDEO) {
            uint32_t first;
            if (dc.env_offset) {
                first = dc.env_offset[e];
            } else {
                uint32_t r[4];
                counter_rng(dc.seed_lo, dc.seed_hi, env, 0xFFFFFFFFu, 2u, 0u, r);
                first = r[0] % dc.n_frames;
            }
            uint32_t clip = 0;  // each environment plays one clip of the set
            if (dc.n_videos > 1) {
                if (dc.env_video) {
                    clip = dc.env_video[e] % dc.n_videos;
                } else {
                    uint32_t r[4];
                    counter_rng(dc.seed_lo, dc.seed_hi, env, 0xFFFFFFFFu, 3u, 0u, r);
                    clip = r[0] % dc.n_videos;
                }
            }
            fu->video_frame = clip * dc.n_frames + (uint32_t)(((u64)first + (u64)step) % dc.n_frames);
        }
    }
    if (VIDEO && sc.lds_vlut) {
        // Video-blend tables: under the clip lies the background or a ground grey (no colour distractor in this
        // mode), so a blended channel is a function of (one of five colours, clip byte).  Four entries per lane.
        // Nine tables of 256 bytes: background r, g, b, then each grey's three times over - the channel of a byte is
        // then the same address offset (256 x channel) whatever lies under the clip, a constant in the read.
        uint32_t* vlut = reinterpret_cast<uint32_t*>(lds + sc.lds_vlut);
        for (uint32_t i = tid; i < 5u * 64u; i += NT) {
            const uint32_t t = i >> 6, at = i & 63u;
            const float c = t == 0 ? sc.bg[0] : t == 1 ? sc.bg[1] : t == 2 ? sc.bg[2] : t == 3 ? sc.gs[0] : sc.gs[1];
            uint32_t word = 0;
#pragma unroll
            for (uint32_t e = 0; e < 4; ++e) {
                const float vf = (float)(at * 4u + e) * (1.0f / 255.0f);
                word |= quantise(__builtin_fmaf(dc.alpha, vf - c, c)) << (8 * e);
            }
            if (t < 3u) {
                vlut[i] = word;
            } else {
                uint32_t* g = vlut + (t == 3u ? 3u * 64u : 6u * 64u) + at;
                g[0] = g[64] = g[128] = word;
            }
        }
    }
    if (tid <= kDrawLane && tid >= kDrawLane - 2u) {
        // Background and the two ground greys are the same for every pixel that shows them: they go through
        // the colour distractor and the quantiser once per frame, one lane per colour.
        const uint32_t k = kDrawLane - tid;
        float scale[3] = {1.0f, 1.0f, 1.0f}, offs[3] = {0.0f, 0.0f, 0.0f};
        if (!VIDEO && dc.mode == PXR_DISTRACT_COLOR) {
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                scale[c] = fu->scale[c];
                offs[c] = fu->offs[c];
            }
        }
        uint32_t packed = 0;
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            float v = k == 0u ? sc.bg[c] : (k == 1u ? sc.gs[0] : sc.gs[1]);
            if (!VIDEO && dc.mode == PXR_DISTRACT_COLOR) {
                v = __builtin_fmaf(v, scale[c], offs[c]);
                v = v > 0.0f ? v : 0.0f;
                v = v < 1.0f ? v : 1.0f;
            }
            fu->base_col[k][c] = v;
            packed |= quantise(v) << (8 * c);
        }
        fu->base_packed[k] = packed;
        if (k == 0u && (VIDEO || dc.mode != PXR_DISTRACT_COLOR)) {
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                fu->scale[c] = 1.0f;
                fu->offs[c] = 0.0f;
            }
        }
    }
    PXR_TIMED_BARRIER(0);
    PXR_PHASE_MARK(0);

    // ---- phase 1: instancing + projection + snap + cell code (one lane per template vertex)
    const bool recip_long_form = !(sc.z_near >= kRecipMin);
    if (tid == NT - 1) vm[sc.V] = 0u;  // the code that the padding of the pair table points at: no pixel centre on either axis
    for (uint32_t v = tid; v < sc.V; v += NT) {
        float pvx, pvy, pvz;
        view_position(sc, v, pvx, pvy, pvz);
        // 1 / pvz is only used when pvz >= z_near (otherwise the vertex is behind the plane or unusable
        // whatever it is), so the short form serves unless some lane's depth is beyond its range
        float inv;
        if (__builtin_expect(recip_long_form || __ballot(pvz > kRecipMax) != 0ull, 0))
            inv = 1.0f / pvz;
        else
            inv = recip_in_range(pvz);
        const float sx = __builtin_fmaf(sc.f, pvx * inv, sc.halfW);
        const float sy = __builtin_fmaf(-sc.f, pvy * inv, sc.halfH);
        const bool ok = (pvz >= sc.z_near) && (__builtin_fabsf(sx) <= 16384.0f) && (__builtin_fabsf(sy) <= 16384.0f);
        // (worked out for every lane, whatever sx and sy are, and replaced where the vertex is not usable: such
        // vertices are rare, and a wavefront without one skips the replacement altogether)
        int X = floor_to_int(__builtin_fmaf(sx, 256.0f, 0.5f));
        int Y = floor_to_int(__builtin_fmaf(sy, 256.0f, 0.5f));
        uint32_t m = cell_code(X, (int)sc.W) | (cell_code(Y, (int)sc.H) << 16);
        if (__builtin_expect(__ballot(!ok) != 0ull, 0)) {
            if (!ok) {
                X = pvz < sc.z_near ? kBehindX : kRejectedX;
                Y = 0;
                m = 0xFFFFFFFFu;  // an unusable or clipped vertex never lets a triangle be discarded early
            }
        }
        vxy[v] = make_int2(X, Y);
        vd[v] = sc.z_near * inv;
        vm[v] = m;
    }
    // (phase 2a's first table entry depends on nothing in LDS: requested before the barrier, it arrives while the
    // wavefront waits there; later ones are requested a trip ahead)
    const uint32_t wave_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid & ~63u));
    uint4 rec_next = make_uint4(0u, 0u, 0u, 0u);
    if (wave_first < sc.P) rec_next = reinterpret_cast<const uint4*>(sc.pair_tbl)[wave_first + lane];
    PXR_TIMED_BARRIER(1);
    PXR_PHASE_MARK(1);

    // ---- phase 2a: coarse binning, one lane per pair of edge-sharing triangles (q0,q1,q2), (q0,q2,q3).
    // A triangle can hold a pixel centre only if, on both axes, its vertices' cell codes are not all
    // equal-and-even; the xor of the codes tells (low half = x, high half = y).
    // The device table is padded to whole wavefronts with entries whose four addresses are those of a word that holds
    // code 0 (never a candidate), so no lane needs a bounds test, and a wavefront past the end leaves.  "Both halves
    // non-zero" is one 16 x 16-bit product; the ballots are taken from single comparisons (their masks as they
    // are) and combined as scalars.
    // (Two trips per turn of the loop, the two entries in flight changing roles: a single "next" variable costs six
    // register moves per trip.)
    const auto coarse_trip = [&](const uint4 rec) {
        const uint32_t w0 = rec.x, w1 = rec.y, w2 = rec.z;
        const uint32_t m0 = lds_u32_at(w0 & 0xFFFFu), m1 = lds_u32_at(w0 >> 16), m2 = lds_u32_at(w1 & 0xFFFFu), m3 = lds_u32_at(w1 >> 16);
        const uint32_t odd = m0 & 0x00010001u, x02 = m0 ^ m2;
        const uint32_t da = (m0 ^ m1) | x02 | odd, db = x02 | (m0 ^ m3) | odd;
        const uint32_t ta = w2 & 0xFFFFu, tb = w2 >> 16;
        const bool keep_a = halves_product(da) != 0u;
        const bool both_b = halves_product(db) != 0u, has_b = tb != kNoTriangle;
        const bool keep_b = both_b && has_b;
        const u64 ma = __ballot(keep_a), mb = __ballot(both_b) & __ballot(has_b);
        if (ma | mb) {
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&fu->n_cand, (uint32_t)(__popcll(ma) + __popcll(mb)));
            base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
            // (the first triangles of the wavefront's entries, then the second ones: the order is free)
            if (keep_a) cand[base + lanes_below(ma)] = (uint16_t)ta;
            if (keep_b) cand[base + (uint32_t)__popcll(ma) + lanes_below(mb)] = (uint16_t)tb;
        }
    };
    {
        const uint4* table = reinterpret_cast<const uint4*>(sc.pair_tbl);
        uint4 rec_a = rec_next, rec_b = make_uint4(0u, 0u, 0u, 0u);
        for (uint32_t p0 = wave_first; p0 < sc.P; p0 += 2 * NT) {
            if (p0 + NT < sc.P) rec_b = table[p0 + NT + lane];
            coarse_trip(rec_a);
            if (p0 + NT >= sc.P) break;
            if (p0 + 2 * NT < sc.P) rec_a = table[p0 + 2 * NT + lane];
            coarse_trip(rec_b);
        }
    }
    PXR_TIMED_BARRIER(2);
    PXR_PHASE_MARK(2);

    // ---- phase 2b: exact binning, one lane per candidate triangle: reject, area sign, pixel range,
    // then one of three bins by the number of candidate pixel centres (one packed LDS atomic per wave).
    const uint32_t n_cand = fu->n_cand;
    // (Where the candidates take several trips - smaller workgroups, taller frames - a lane's candidate and its entry
    // of the index table are requested a trip ahead, without a branch: a lane past the end reads a list entry that
    // nobody wrote and clamps it into the table.  The 1024-thread unbanded kernel sees its ~900 candidates in one trip
    // and is bound by instruction issue: it keeps the plain form.)
    constexpr bool kAhead = NT < 1024 || BANDED;
    uint32_t t_ahead = 0;
    uint2 ti_ahead = make_uint2(0u, 0u);
    if (kAhead) {
        t_ahead = cand[min(tid, sc.T - 1u)];
        ti_ahead = reinterpret_cast<const uint2*>(sc.tri_idx)[min(t_ahead, sc.T - 1u)];
    }
    for (uint32_t k0 = 0; k0 < n_cand; k0 += NT) {
        const uint32_t k = k0 + tid;
        int cls = 0;  // 0 none, 1 tiny, 2 small, 3 large
        uint32_t t = t_ahead;
        uint2 ti = ti_ahead;
        if (kAhead) {
            if (k0 + NT < n_cand) {
                t_ahead = cand[min(k + NT, sc.T - 1u)];
                ti_ahead = reinterpret_cast<const uint2*>(sc.tri_idx)[min(t_ahead, sc.T - 1u)];
            }
        } else if (k < n_cand) {
            t = cand[k];
            ti = reinterpret_cast<const uint2*>(sc.tri_idx)[t];
        }
        if (k < n_cand) {
            TriSetup s;
            uint32_t v0, v1, v2;
            bool small_extent;
            const int kind = tri_gather(sc, ti, vxy, s, v0, v1, v2, small_extent);
            if (kind == kTriClip) cls = 3;  // clipped, then rastered, by a whole wavefront
            if (kind == kTriPlain) {
                bool front;
                if (small_extent)
                    front = __mul24(s.bx - s.ax, s.cy - s.ay) > __mul24(s.by - s.ay, s.cx - s.ax);
                else
                    front = (long long)(s.bx - s.ax) * (long long)(s.cy - s.ay) >
                            (long long)(s.by - s.ay) * (long long)(s.cx - s.ax);
                if (front) {
                    const uint32_t npx = __umul24((uint32_t)(s.i1 - s.i0 + 1), (uint32_t)(s.j1 - s.j0 + 1));  // (each at most 512)
                    cls = npx <= kTinyMaxPixels ? 1 : (npx <= kSmallMaxPixels ? 2 : 3);
                }
            }
        }
        const u64 m1 = __ballot(cls == 1), m2 = __ballot(cls == 2), m3 = __ballot(cls == 3);
        if (m1 | m2 | m3) {
            u64 old = 0;
            if (lane == 0)
                old = atomicAdd(&fu->bins, (u64)__popcll(m1) | ((u64)__popcll(m2) << 16) | ((u64)__popcll(m3) << 32));
            const uint32_t old_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)old);
            const uint32_t old_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(old >> 32));
            if (cls == 1) list[(old_lo & 0xFFFFu) + lanes_below(m1)] = (uint16_t)t;
            if (cls == 2) list[sc.T - 1 - ((old_lo >> 16) + lanes_below(m2))] = (uint16_t)t;
            if (cls == 3) list2[old_hi + lanes_below(m3)] = (uint16_t)t;
        }
    }
    PXR_TIMED_BARRIER(3);
    PXR_PHASE_MARK(3);

    // Tall frames are rendered in horizontal bands so that the key buffer stays small enough for two
    // workgroups per compute unit; geometry work (phases 0-2) is done once, raster and resolve per band.
    uint32_t row_lo = 0;
    uint32_t band_round = 0;  // banded frames: rounds of the band-list builder so far (picks the counter slot)
    const uint32_t tid_kept = tid;
    do {
        const SceneConsts& scb = BANDED ? argument_reloaded<SceneConsts>(kSceneArgAt) : sc;
        const DistractConsts& dcb = BANDED ? argument_reloaded<DistractConsts>(kDistractArgAt) : dc;
        // (In the band loop everything is derived again from the reloaded arguments and from a thread index the
        // compiler cannot see through: nothing but the row counter and the index stays live from band to band.)
        uint32_t tid = tid_kept;
        if (BANDED) asm volatile("" : "+v"(tid));
        const uint32_t lane = tid & 63u;
        u64* keys = reinterpret_cast<u64*>(lds + scb.lds_keys);
        int2* vxy = reinterpret_cast<int2*>(lds + scb.lds_vxy);
        float* vd = reinterpret_cast<float*>(lds + scb.lds_vd);
        float* body = reinterpret_cast<float*>(lds + scb.lds_body);
        float* cxcy = reinterpret_cast<float*>(lds + scb.lds_cxcy);
        float4* rows = reinterpret_cast<float4*>(lds + scb.lds_rows);
        FrameUniforms* fu = reinterpret_cast<FrameUniforms*>(lds + scb.lds_misc);
        uint16_t* list = reinterpret_cast<uint16_t*>(lds + scb.lds_list);
        uint16_t* list2 = reinterpret_cast<uint16_t*>(lds + scb.lds_large);
        const uint32_t row_hi = BANDED ? min(scb.H, row_lo + (row_lo ? scb.band_rows : scb.first_band_rows)) : scb.H;
        const uint32_t p_begin = row_lo * scb.W, p_end = row_hi * scb.W;
        // keys to clear before the first band: all the buffer holds (a later band may be taller than the first, and
        // every lane only leaves the keys it resolved cleared)
        const uint32_t n_keys = BANDED ? scb.band_rows * scb.W : p_end - p_begin;
        if (!BANDED || scb.lds_blist == 0) {
            // Unbanded frames, and frames of a few bands (every band walks all bins: cheaper than picking a band's
            // triangles out while a triangle's rows are looked at by two or three bands only).
            if (BANDED && row_lo) __syncthreads();  // the previous band is resolved (its lanes left their keys cleared)
            // The bins are complete: each lane asks now for the first triangle it will raster from the small and from the
            // tiny bin (its list entry, then its entry of the index table), so that they come in from memory while the keys
            // are cleared and the barrier is waited at.
            const u64 bins = fu->bins;
            const uint32_t n_tiny = (uint32_t)bins & 0xFFFFu, n_small = (uint32_t)bins >> 16, n_large = (uint32_t)(bins >> 32);
            constexpr uint32_t kTeam = 1u << kSmallLanesLog2;
            const uint2* tri_table = reinterpret_cast<const uint2*>(scb.tri_idx);
            // (Asked for without a branch, so that nothing has to wait for the answers here: a lane with no triangle in a
            // bin reads a list entry that may never have been written and clamps it into the table.)
            uint32_t t_small = list[scb.T - 1 - min(tid >> kSmallLanesLog2, scb.T - 1u)];
            uint32_t t_tiny = list[min(NT - 1 - tid, scb.T - 1u)];
            uint2 ti_small = tri_table[min(t_small, scb.T - 1u)], ti_tiny = tri_table[min(t_tiny, scb.T - 1u)];

            // codes and candidates are dead: clear the pixel keys they shared LDS with (0 = background at depth 0)
            // (two keys per store; the region is padded to 16 bytes, so an odd count may clear one key more)
            if (!BANDED || row_lo == 0) {
                for (uint32_t p = tid; p < (n_keys + 1u) >> 1; p += NT)
                    reinterpret_cast<uint4*>(keys)[p] = make_uint4(0u, 0u, 0u, 0u);
                PXR_TIMED_BARRIER(4);
            }
            PXR_PHASE_MARK(4);

            // ---- phase 3: raster + z-test into the LDS key buffer.  The bins start at different
            // lanes of the workgroup so that all waves get a share.
            // The hardware favours a workgroup's older wavefronts when several want to issue, so the youngest finish a
            // phase last: the heavier bin goes to the oldest.
            // small: a team of lanes per triangle, from the first lane up
            // (a lane's first triangle of each was requested before the barrier; the next one is at the loop's end)
            for (uint32_t k = tid >> kSmallLanesLog2; k < n_small;) {
                raster_binned<false>(scb, t_small, ti_small, vxy, vd, keys, (int)(tid & (kTeam - 1u)), (int)kSmallLanesLog2,
                                     (int)row_lo, (int)row_hi);
                k += NT >> kSmallLanesLog2;
                if (k < n_small) {
                    t_small = list[scb.T - 1 - k];
                    ti_small = tri_table[t_small];
                }
            }
            // tiny: one lane per triangle, from the last lane down
            for (uint32_t k = NT - 1 - tid; k < n_tiny;) {
                raster_binned<false>(scb, t_tiny, ti_tiny, vxy, vd, keys, 0, 0, (int)row_lo, (int)row_hi);
                k += NT;
                if (k < n_tiny) {
                    t_tiny = list[k];
                    ti_tiny = tri_table[t_tiny];
                }
            }
            // large: a whole wave per triangle, starting in the middle waves
            for (uint32_t k = ((tid >> 6) + NT / 128) % (NT / 64); k < n_large; k += NT / 64)
                raster_binned<true>(scb, list2[k], tri_table[list2[k]], vxy, vd, keys, (int)lane, 6, (int)row_lo, (int)row_hi);
            PXR_TIMED_BARRIER(5);
            PXR_PHASE_MARK(5);

        } else {
            // Frames of many bands.  Every band walks the frame's bins again, but only to pick out the triangles that can
            // touch its rows: a dense pass, one lane per binned triangle and round of NT, that compacts them (ballot,
            // one packed atomic per wavefront) into the round's own short lists, from which the raster loops then
            // work as in the unbanded kernel.  A band that holds a twentieth of the frame's triangles rasters a
            // twentieth of them, not all.
            if (row_lo) __syncthreads();  // the previous band is resolved (its lanes left their keys cleared)
            uint16_t* blist = reinterpret_cast<uint16_t*>(lds + scb.lds_blist);    // tiny up, small down: kBandListEntries
            uint16_t* blist2 = reinterpret_cast<uint16_t*>(lds + scb.lds_blist2);  // large: kBandListEntries
            const u64 bins = fu->bins;
            const uint32_t n_tiny = (uint32_t)bins & 0xFFFFu, n_small = (uint32_t)bins >> 16, n_large = (uint32_t)(bins >> 32);
            const uint32_t n_binned = n_tiny + n_small + n_large;
            constexpr uint32_t kTeam = 1u << kSmallLanesLog2;
            const uint2* tri_table = reinterpret_cast<const uint2*>(scb.tri_idx);
            if (row_lo == 0) {
                // the first band's keys share LDS with the cell codes and the candidate list, dead by now
                for (uint32_t p = tid; p < (n_keys + 1u) >> 1; p += NT)
                    reinterpret_cast<uint4*>(keys)[p] = make_uint4(0u, 0u, 0u, 0u);
            }
            uint32_t base = 0;
            do {
                // ---- this round's share of the bins -> the triangles among them that touch rows [row_lo, row_hi)
                const uint32_t slot = band_round & 1u;
                if (tid == 0) fu->band_bins[slot ^ 1u] = 0ull;  // (last read before the barrier that ended the round before this one)
                const uint32_t k = base + tid;
                int cls = 0;
                uint32_t t = 0;
                if (k < n_binned) {
                    cls = k < n_tiny ? 1 : (k < n_tiny + n_small ? 2 : 3);
                    t = cls == 1 ? list[k] : (cls == 2 ? list[scb.T - 1 - (k - n_tiny)] : list2[k - n_tiny - n_small]);
                    int j0 = 0, j1 = 0;
                    if (tri_rows(scb, tri_table[t], vxy, j0, j1) == kTriPlain && (j0 >= (int)row_hi || j1 < (int)row_lo)) cls = 0;
                }
                const u64 m1 = __ballot(cls == 1), m2 = __ballot(cls == 2), m3 = __ballot(cls == 3);
                if (m1 | m2 | m3) {
                    u64 old = 0;
                    if (lane == 0)
                        old = atomicAdd(&fu->band_bins[slot], (u64)__popcll(m1) | ((u64)__popcll(m2) << 16) | ((u64)__popcll(m3) << 32));
                    const uint32_t old_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)old);
                    const uint32_t old_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(old >> 32));
                    // (a round looks at NT triangles: tiny and small together never outgrow the NT entries they share)
                    if (cls == 1) blist[(old_lo & 0xFFFFu) + lanes_below(m1)] = (uint16_t)t;
                    if (cls == 2) blist[kBandListEntries - 1 - ((old_lo >> 16) + lanes_below(m2))] = (uint16_t)t;
                    if (cls == 3) blist2[old_hi + lanes_below(m3)] = (uint16_t)t;
                }
                PXR_TIMED_BARRIER(4);
                PXR_PHASE_MARK(4);

                // ---- phase 3 from the round's lists (lane teams as in the unbanded kernel)
                const u64 bb = fu->band_bins[slot];
                const uint32_t b_tiny = (uint32_t)bb & 0xFFFFu, b_small = (uint32_t)bb >> 16, b_large = (uint32_t)(bb >> 32);
                for (uint32_t i = tid >> kSmallLanesLog2; i < b_small; i += NT >> kSmallLanesLog2) {
                    const uint32_t ts = blist[kBandListEntries - 1 - i];
                    raster_binned<false>(scb, ts, tri_table[ts], vxy, vd, keys, (int)(tid & (kTeam - 1u)), (int)kSmallLanesLog2,
                                         (int)row_lo, (int)row_hi);
                }
                if (NT - 1 - tid < b_tiny) {
                    const uint32_t tt = blist[NT - 1 - tid];
                    raster_binned<false>(scb, tt, tri_table[tt], vxy, vd, keys, 0, 0, (int)row_lo, (int)row_hi);
                }
                for (uint32_t i = ((tid >> 6) + NT / 128) % (NT / 64); i < b_large; i += NT / 64)
                    raster_binned<true>(scb, blist2[i], tri_table[blist2[i]], vxy, vd, keys, (int)lane, 6, (int)row_lo, (int)row_hi);
                PXR_TIMED_BARRIER(5);
                PXR_PHASE_MARK(5);
                ++band_round;
                base += NT;
            } while (base < n_binned);
        }

        // ---- phase 4: resolve + shade + distractor + pack + store
        ResolveCtx rc;
        const float eye_x = fu->eye[0], eye_y = fu->eye[1], eye_z = fu->eye[2];
        rc.eye_x = eye_x;
        rc.eye_y = eye_y;
        rc.eye_z = eye_z;
        const bool no_roll = scb.Rt[2] == 0.0f;
        rc.inv_ez = 0.0f;
        if (!(PX == 4 && no_roll)) {  // (without roll the row table already holds the ground test)
            asm volatile("" ::: "memory");  // (a branch, not a select: the compiler would do the division either way)
            rc.inv_ez = 1.0f / eye_z;
        }
        rc.ground_ok = scb.ground_on && eye_z > 0.0f;
        rc.mode = dcb.mode;
        rc.alpha = dcb.alpha;
        rc.vframe = nullptr;
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            rc.scale[c] = fu->scale[c];
            rc.offs[c] = fu->offs[c];
        }
        rc.col_addr = scb.lds_misc + (uint32_t)offsetof(FrameUniforms, base_col);
        rc.packed_addr = scb.lds_misc + (uint32_t)offsetof(FrameUniforms, base_packed);
        rc.vlut = scb.lds_vlut;
        if (VIDEO) rc.vframe = dcb.video + (size_t)fu->video_frame * scb.npix * 3;
        uint8_t* out = frames + (size_t)frame * scb.npix * 3;
        uint32_t* out_ids = ids ? ids + (size_t)frame * scb.npix : nullptr;
        if (PX == 4) {
            // uniform scene properties select a specialised loop (kept out of the per-pixel code)
            // (an eye that is a NaN makes ground points NaNs: such a frame takes the general loop, which is exact
            // for a unit cell as well)
            if (scb.checker_short_form && eye_x == eye_x && eye_y == eye_y) {
                if (no_roll)
                    resolve_rows4<NT, true, true, VIDEO, BANDED>(scb, rc, body, cxcy, rows, keys, out, out_ids, tid, p_begin, p_end);
                else
                    resolve_rows4<NT, true, false, VIDEO, BANDED>(scb, rc, body, cxcy, rows, keys, out, out_ids, tid, p_begin, p_end);
            } else {
                if (no_roll)
                    resolve_rows4<NT, false, true, VIDEO, BANDED>(scb, rc, body, cxcy, rows, keys, out, out_ids, tid, p_begin, p_end);
                else
                    resolve_rows4<NT, false, false, VIDEO, BANDED>(scb, rc, body, cxcy, rows, keys, out, out_ids, tid, p_begin, p_end);
            }
        } else {
            // any image shape: one pixel per lane, byte stores
            for (uint32_t p = p_begin + tid; p < p_end; p += NT) {
                const uint32_t j = __umulhi(p, scb.magicW);
                const uint32_t i = p - j * scb.W;
                const float cxi = cxcy[i], cyj = cxcy[scb.W + j];
                const float dwx = __builtin_fmaf(scb.Rt[0], cxi, __builtin_fmaf(scb.Up[0], cyj, scb.Fw[0]));
                const float dwy = __builtin_fmaf(scb.Rt[1], cxi, __builtin_fmaf(scb.Up[1], cyj, scb.Fw[1]));
                const float dwz = __builtin_fmaf(scb.Rt[2], cxi, __builtin_fmaf(scb.Up[2], cyj, scb.Fw[2]));
                float tg;
                const u64 gkey = ground_key(scb, rc, -dwz, tg);
                uint32_t vbytes = 0;
                if (VIDEO) {
                    const uint8_t* v = rc.vframe + (size_t)p * 3;
                    vbytes = (uint32_t)v[0] | ((uint32_t)v[1] << 8) | ((uint32_t)v[2] << 16);
                }
                uint32_t low;
                u64 unused;
                const uint32_t rgb = resolve_pixel<false, VIDEO>(scb, rc, body, keys[p - p_begin], gkey, tg, dwx, dwy, vbytes, low, unused);
                out[(size_t)p * 3 + 0] = (uint8_t)(rgb & 0xFFu);
                out[(size_t)p * 3 + 1] = (uint8_t)((rgb >> 8) & 0xFFu);
                out[(size_t)p * 3 + 2] = (uint8_t)(rgb >> 16);
                if (out_ids) out_ids[p] = 0xFFFFFFFFu - low;
                if (BANDED) keys[p - p_begin] = 0ull;  // cleared for the next band by the lane that read it
            }
        }
        row_lo = row_hi;
    } while (BANDED && row_lo < argument_reloaded<SceneConsts>(kSceneArgAt).H);
    PXR_PHASE_MARK(6);
    PXR_PHASE_END();
}

template <int NT, int PX, bool BANDED, bool VIDEO>
int launch_one(const SceneConsts& sc, const DistractConsts& dc, const float* d_poses, const float* d_shapes,
               uint32_t n_frames, uint32_t S, uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids,
               hipStream_t stream, std::string& err) {
    hipLaunchKernelGGL((render_kernel<NT, PX, BANDED, VIDEO>), dim3(n_frames), dim3(NT), sc.lds_total, stream, sc, dc,
                       d_poses, d_shapes, S, step0, env0, d_frames, d_ids);
    const hipError_t rc = hipGetLastError();
    if (rc != hipSuccess) {
        err = std::string("kernel launch failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

template <int NT, int PX, bool BANDED, bool VIDEO>
int prepare_one(uint32_t lds_bytes, std::string& err) {
    hipFuncAttributes attr;
    if (hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&render_kernel<NT, PX, BANDED, VIDEO>)) != hipSuccess ||
        attr.sharedSizeBytes != 0) {
        err = "the render kernel has static LDS in front of its dynamic segment (LDS addresses in the tables assume none)";
        return PXR_ERR_DEVICE;
    }
    const hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&render_kernel<NT, PX, BANDED, VIDEO>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (rc != hipSuccess) {
        err = std::string("hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

template <int NT>
int prepare_all(uint32_t cap, std::string& err) {
    int rc;
    if ((rc = prepare_one<NT, 4, false, false>(cap, err))) return rc;
    if ((rc = prepare_one<NT, 4, true, false>(cap, err))) return rc;
    if ((rc = prepare_one<NT, 1, false, false>(cap, err))) return rc;
    if ((rc = prepare_one<NT, 1, true, false>(cap, err))) return rc;
    if ((rc = prepare_one<NT, 4, false, true>(cap, err))) return rc;
    if ((rc = prepare_one<NT, 4, true, true>(cap, err))) return rc;
    if ((rc = prepare_one<NT, 1, false, true>(cap, err))) return rc;
    if ((rc = prepare_one<NT, 1, true, true>(cap, err))) return rc;
    return PXR_OK;
}

#if defined(PXR_PROFILING_BUILD) && defined(PXR_PHASE_TIMING)
#include "profiling/phase_exports.h"
#endif

}  // namespace

int prepare_kernels(std::string& err) {
    // The attribute is a per-kernel cap, not a per-launch size: raise it to the whole 160 KB, so that scenes
    // of any size can coexist.
    const uint32_t cap = 160u * 1024u;
    int rc;
    if ((rc = prepare_all<256>(cap, err))) return rc;
    if ((rc = prepare_all<512>(cap, err))) return rc;
    if ((rc = prepare_all<768>(cap, err))) return rc;
    if ((rc = prepare_all<1024>(cap, err))) return rc;
    return PXR_OK;
}

int launch_render(const SceneConsts& sc, const DistractConsts& dc, const float* d_poses, const float* d_shapes,
                  uint32_t n_frames, uint32_t S, uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids,
                  uint32_t block_threads, void* stream, std::string& err) {
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // four pixels per lane: they must share a row and frames must stay dword-aligned
    const bool quad = (sc.W % 4u) == 0u;
    const bool banded = sc.band_rows < sc.H;
    // (the video distractor has kernels of its own: the others carry none of its code, and the other way round)
    const bool video = dc.mode == PXR_DISTRACT_VIDEO;
#define PXR_ARGS sc, dc, d_poses, d_shapes, n_frames, S, step0, env0, d_frames, d_ids, st, err
#define PXR_LAUNCH_V(NT, V)                                                                            \
    return quad ? (banded ? launch_one<NT, 4, true, V>(PXR_ARGS) : launch_one<NT, 4, false, V>(PXR_ARGS)) \
                : (banded ? launch_one<NT, 1, true, V>(PXR_ARGS) : launch_one<NT, 1, false, V>(PXR_ARGS))
#define PXR_LAUNCH(NT)                   \
    if (video) PXR_LAUNCH_V(NT, true);   \
    PXR_LAUNCH_V(NT, false)
    switch (block_threads) {
        case 256: PXR_LAUNCH(256);
        case 512: PXR_LAUNCH(512);
        case 768: PXR_LAUNCH(768);
        case 1024: PXR_LAUNCH(1024);
        default:
            err = "block_threads must be 256, 512, 768 or 1024";
            return PXR_ERR_INVALID_ARG;
    }
#undef PXR_LAUNCH
#undef PXR_LAUNCH_V
#undef PXR_ARGS
}

}  // namespace pxr
