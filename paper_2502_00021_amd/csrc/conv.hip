// Frame consumer of libpxr: the policy's first convolutional layer applied to
// the rendered frame stack, straight from the uint8 frames (PixelBrax, arXiv
// 2502.00021, section 2: every environment step of the paper's throughput loop
// ends in a forward pass through one convolutional layer).  gfx950 only.
//
//   out[b,oy,ox,o] = act(bias[o] + sum_{ky,kx,s,c} frames[b,s,2oy+ky,2ox+kx,c]/255 * w[ky,kx,3s+c,o])
//
// 3x3 kernel, stride 2, no padding, 32 output channels, bf16 weights, fp32
// accumulation, bf16 NHWC output.  This IS a dense contraction (per
// environment a [Ho*Wo x 27S] x [27S x 32] product), so it runs on the matrix
// cores (v_mfma_f32_32x32x16_bf16), but at ~50 FLOP per byte of HBM traffic it
// is bound by HBM: the design goal is one read of every frame byte, one full
// 64-byte-line write of every output pixel, and nothing else.
//
// Work item = (environment, band of output rows).  Workgroups are persistent
// (the 36 registers of weights per lane are loaded once per wave) and walk the
// items with a grid stride:
//   load   the band's input rows of all S frames: 12-byte loads (4 RGB pixels),
//          issued one work item ahead into registers, then uint8 -> bf16
//          (exact) and written to LDS as [frame][row][pixel][R,G,B,0]
//   mma    one wavefront per (output row, 32-pixel tile): for each (frame, ky)
//          ONE aligned 16-byte LDS read per lane is the B operand
//          (2 pixels x 4 channels; lanes 0-31 take pixels 2ox, 2ox+1, lanes
//          32-63 take 2ox+2, 2ox+3; the weights of pixel 2ox+3 and of channel 3
//          are zero), A = the weights: 3S instructions per tile
//   store  fma(acc, 1/255, bias), ReLU, bf16 (round to nearest even), staged
//          through 2 KB of wave-private LDS so that a tile leaves as two
//          contiguous 1 KB stores
// Matrix rows are permuted so that each lane ends up with 16 consecutive
// output channels of its pixel (row 8a + 4g + b holds channel 16g + 4a + b).

#include <hip/hip_runtime.h>

#include "pxr_internal.h"

namespace pxr {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kConvThreads = 256;
constexpr uint32_t kStageBytes = 2048;  // per wave: 32 pixels x 32 channels x bf16
constexpr uint32_t kConvTrips = 4;      // 12-byte input quads a thread carries per work item

// float(n) for a byte n has at most 8 significant bits: its upper half IS bfloat16(n).
__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi) {
    return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
}

__device__ __forceinline__ uint32_t to_bf16_pair(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // v_cvt_pk_bf16_f32: round to nearest even
}

// Streaming 16-byte store, written as an instruction so that the compiler's wait-count pass does not see a
// vector-memory operation inside the per-tile loop: with a visible store there it drains the memory counter
// before entering the loop, which would make every wave sit out the latency of the loads just issued for the
// next work item instead of covering it with the matrix work.  (The counter is shared by loads and stores and
// only ever over-waited by this: a later wait for "at most n operations outstanding" still implies that the
// older loads have returned.)
// The two idle cycles after it are the ones the hardware asks for between a store of more than 8 bytes and a
// vector instruction that overwrites the stored registers; the compiler adds them for stores it can see.
__device__ __forceinline__ void store_streaming_b128(void* dst, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off nt\n\ts_nop 1" : : "v"(dst), "v"(v) : "memory");
}

template <int S, bool RELU>
__global__ __launch_bounds__(kConvThreads) void conv_kernel(const ConvConsts cc, const uint8_t* __restrict__ frames,
                                                            uint32_t n_items, uint16_t* __restrict__ out) {
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t g = lane >> 5, n = lane & 31u;
    const uint32_t frame_lds = cc.rows_in * cc.W * 8u;  // bytes of one frame's band in LDS
    unsigned char* stage = lds + S * frame_lds + wave * kStageBytes;

    // per-wave constants: the A operands and this lane's 16 biases
    bf16x8 aw[3 * S];
#pragma unroll
    for (int j = 0; j < 3 * S; ++j) {
        const uint4 v = reinterpret_cast<const uint4*>(cc.wtab)[j * 64 + lane];
        aw[j] = __builtin_bit_cast(bf16x8, v);
    }
    float bias[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bias[i] = cc.bias[16 * g + i];
    // Let the weights arrive before the first input request goes out: the memory counter is in-order, so a
    // later wait that has to cover a possibly pending weight register would also wait for every prefetched
    // input behind it, in every tile of every work item.  (s_waitcnt vmcnt(0); other counters untouched.)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");

    // A work item's input: rows 2*oy0 .. 2*oy0 + rows - 1 of each of the S frames, as "quads" of 4 pixels
    // (12 bytes).  Quad f of the item (f = tid + 256 p) belongs to frame s = f / n_quads.  An item's quads
    // are fetched into registers one item ahead, so that HBM latency hides behind the previous item's
    // matrix work; the host guarantees S * n_quads <= 256 * kConvTrips.
    struct alignas(4) Quad {
        uint32_t a, b, c;
    };
    Quad pre[kConvTrips];
    const uint32_t quads_per_row = cc.W >> 2;
    auto fetch = [&](uint32_t item) {
        const uint32_t env = item / cc.bands, oy0 = (item - env * cc.bands) * cc.band_rows;
        const uint32_t n_quads = (2u * min(cc.band_rows, cc.Ho - oy0) + 1u) * quads_per_row;
        // (an environment's S frames are at most 1.5 MB: offsets inside them fit 32 bits)
        const unsigned char* base = frames + (size_t)env * (S * cc.H * cc.W * 3u) + 2u * oy0 * cc.W * 3u;
        const uint32_t frame_bytes = cc.H * cc.W * 3u;
        // Unconditional loads (lanes past the item's last quad re-read it): with no branch around them the four
        // requests of a thread are in flight together; a guarded load makes the compiler wait for the previous
        // one before it reuses the guard's registers.
#pragma unroll
        for (uint32_t p = 0; p < kConvTrips; ++p) {
            const uint32_t f = min(tid + p * kConvThreads, S * n_quads - 1u);
            uint32_t s = 0, q = f;
#pragma unroll
            for (int t = 1; t < S; ++t)
                if (f >= t * n_quads) {
                    s = t;
                    q = f - t * n_quads;
                }
            pre[p] = *reinterpret_cast<const Quad*>(base + (s * frame_bytes + q * 12u));
        }
    };

    uint32_t item = blockIdx.x;
    if (item < n_items) fetch(item);
    while (item < n_items) {
        const uint32_t env = item / cc.bands, band = item - env * cc.bands;
        const uint32_t oy0 = band * cc.band_rows;
        const uint32_t rows_out = min(cc.band_rows, cc.Ho - oy0);
        const uint32_t n_quads = (2u * rows_out + 1u) * quads_per_row;

        // ---- convert the fetched quads to bf16 and lay them out in LDS
#pragma unroll
        for (uint32_t p = 0; p < kConvTrips; ++p) {
            const uint32_t f = tid + p * kConvThreads;
            uint32_t s = 0, q = f;
#pragma unroll
            for (int t = 1; t < S; ++t)
                if (f >= t * n_quads) {
                    s = t;
                    q = f - t * n_quads;
                }
            if (f < S * n_quads) {
                const uint32_t d0 = pre[p].a, d1 = pre[p].b, d2 = pre[p].c;
                const float r0 = (float)(d0 & 0xFFu), g0 = (float)((d0 >> 8) & 0xFFu), b0 = (float)((d0 >> 16) & 0xFFu);
                const float r1 = (float)(d0 >> 24), g1 = (float)(d1 & 0xFFu), b1 = (float)((d1 >> 8) & 0xFFu);
                const float r2 = (float)((d1 >> 16) & 0xFFu), g2 = (float)(d1 >> 24), b2 = (float)(d2 & 0xFFu);
                const float r3 = (float)((d2 >> 8) & 0xFFu), g3 = (float)((d2 >> 16) & 0xFFu), b3 = (float)(d2 >> 24);
                uint4* o = reinterpret_cast<uint4*>(lds + s * frame_lds + (size_t)q * 32u);
                o[0] = make_uint4(bf16_pair(r0, g0), __float_as_uint(b0) >> 16, bf16_pair(r1, g1), __float_as_uint(b1) >> 16);
                o[1] = make_uint4(bf16_pair(r2, g2), __float_as_uint(b2) >> 16, bf16_pair(r3, g3), __float_as_uint(b3) >> 16);
            }
        }
        __syncthreads();
        const uint32_t next = item + gridDim.x;
        if (next < n_items) fetch(next);

        // ---- one wavefront per (output row, 32-pixel tile)
        const uint32_t n_tasks = rows_out * cc.tiles_x;
        for (uint32_t task = wave; task < n_tasks; task += kConvThreads / 64) {
            const uint32_t r_out = __umul24(task, cc.tiles_magic) >> 16, tx = task - __umul24(r_out, cc.tiles_x);  // task / tiles_x
            const uint32_t ox = min(tx * 32u + n, cc.Wo - 1u);  // lanes past the row's end recompute its last pixel
            const unsigned char* bsrc = lds + (__umul24(2u * r_out, cc.W) + 2u * ox + 2u * g) * 8u;
            f32x16 acc = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int s = 0; s < S; ++s)
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) {
                    const uint4 v = *reinterpret_cast<const uint4*>(bsrc + (s * frame_lds + ky * cc.W * 8u));
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aw[s * 3 + ky], __builtin_bit_cast(bf16x8, v), acc, 0, 0, 0);
                }
            uint32_t packed[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float a = __builtin_fmaf(acc[2 * i], 1.0f / 255.0f, bias[2 * i]);
                float b = __builtin_fmaf(acc[2 * i + 1], 1.0f / 255.0f, bias[2 * i + 1]);
                if (RELU) {
                    a = __builtin_fmaxf(a, 0.0f);
                    b = __builtin_fmaxf(b, 0.0f);
                }
                packed[i] = to_bf16_pair(a, b);
            }
            uint4* st = reinterpret_cast<uint4*>(stage + n * 64u + g * 32u);
            st[0] = make_uint4(packed[0], packed[1], packed[2], packed[3]);
            st[1] = make_uint4(packed[4], packed[5], packed[6], packed[7]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const uint32_t n_bytes = min(32u, cc.Wo - tx * 32u) * 64u;
            // (an environment's features are below 2 GB: 32-bit offsets from its base)
            unsigned char* dst = reinterpret_cast<unsigned char*>(out) + (size_t)env * (cc.Ho * cc.Wo * 64u) +
                                 (__umul24(oy0 + r_out, cc.Wo) + tx * 32u) * 64u;
#pragma unroll
            for (uint32_t h = 0; h < 2; ++h) {
                const uint32_t off = h * 1024u + lane * 16u;
                // the features are not read again by this kernel: streaming stores keep them out of the caches' way
                if (off < n_bytes) store_streaming_b128(dst + off, *reinterpret_cast<const u32x4*>(stage + off));
            }
            __builtin_amdgcn_wave_barrier();  // the next tile's staging writes stay behind these reads
        }
        __syncthreads();  // the next item's conversion overwrites the band
        item = next;
    }
}

}  // namespace

uint32_t conv_max_quads() { return kConvThreads * kConvTrips; }

uint32_t conv_lds_bytes(const ConvConsts& cc) {
    return cc.S * cc.rows_in * cc.W * 8u + (kConvThreads / 64u) * kStageBytes;
}

int prepare_conv_kernels(std::string& err) {
    const void* fns[8] = {reinterpret_cast<const void*>(&conv_kernel<1, true>), reinterpret_cast<const void*>(&conv_kernel<2, true>),
                          reinterpret_cast<const void*>(&conv_kernel<3, true>), reinterpret_cast<const void*>(&conv_kernel<4, true>),
                          reinterpret_cast<const void*>(&conv_kernel<1, false>), reinterpret_cast<const void*>(&conv_kernel<2, false>),
                          reinterpret_cast<const void*>(&conv_kernel<3, false>), reinterpret_cast<const void*>(&conv_kernel<4, false>)};
    for (const void* f : fns) {
        const hipError_t rc = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (rc != hipSuccess) {
            err = std::string("hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: ") + hipGetErrorString(rc);
            return PXR_ERR_DEVICE;
        }
    }
    return PXR_OK;
}

int launch_conv(const ConvConsts& cc, const uint8_t* d_frames, uint32_t B, uint16_t* d_out, uint32_t n_groups, void* stream,
                std::string& err) {
    const uint32_t n_items = B * cc.bands;
    const uint32_t grid = min(n_items, n_groups);
    const uint32_t ldsb = conv_lds_bytes(cc);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
#define PXR_CONV_LAUNCH(SS)                                                                                             \
    if (cc.relu)                                                                                                        \
        hipLaunchKernelGGL((conv_kernel<SS, true>), dim3(grid), dim3(kConvThreads), ldsb, st, cc, d_frames, n_items, d_out); \
    else                                                                                                                \
        hipLaunchKernelGGL((conv_kernel<SS, false>), dim3(grid), dim3(kConvThreads), ldsb, st, cc, d_frames, n_items, d_out); \
    break
    switch (cc.S) {
        case 1: PXR_CONV_LAUNCH(1);
        case 2: PXR_CONV_LAUNCH(2);
        case 3: PXR_CONV_LAUNCH(3);
        case 4: PXR_CONV_LAUNCH(4);
        default: err = "frame stack depth must lie in [1,4]"; return PXR_ERR_UNSUPPORTED;
    }
#undef PXR_CONV_LAUNCH
    const hipError_t rc = hipGetLastError();
    if (rc != hipSuccess) {
        err = std::string("kernel launch failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

}  // namespace pxr
