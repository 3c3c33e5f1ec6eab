// C ABI of the frame consumer (pxr_conv_* in include/pxr.h): validation, the
// host-side layout of the weights for the matrix instruction, launch.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>

#include "pxr_internal.h"

struct pxr_conv {
    pxr::ConvConsts cc{};
    void* d_tables = nullptr;
    uint32_t n_groups = 0;       // persistent workgroups per launch
    uint32_t default_band = 0, default_groups = 0;
    uint32_t n_cus = 0;
};

namespace {

// fp32 -> bfloat16 bits, round to nearest, ties to even (input is finite)
uint16_t bf16_rne(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

void plan(pxr_conv* c, uint32_t band_rows) {
    pxr::ConvConsts& cc = c->cc;
    cc.bands = (cc.Ho + band_rows - 1) / band_rows;
    cc.band_rows = (cc.Ho + cc.bands - 1) / cc.bands;  // even out the bands
    cc.bands = (cc.Ho + cc.band_rows - 1) / cc.band_rows;
    cc.rows_in = 2 * cc.band_rows + 1;
}

}  // namespace

void pxr::conv_shape(const pxr_conv* c, uint32_t* H, uint32_t* W, uint32_t* S, uint32_t* Ho, uint32_t* Wo) {
    *H = c->cc.H;
    *W = c->cc.W;
    *S = c->cc.S;
    *Ho = c->cc.Ho;
    *Wo = c->cc.Wo;
}

int pxr::conv_envs(pxr_conv* c, const uint8_t* d_frames, uint32_t e0, uint32_t n, uint16_t* d_out, void* stream, std::string& err) {
    if (n == 0 || (uint64_t)n * c->cc.bands > 0x7FFFFFFFull) {
        err = "B must be positive and B * bands below 2^31";
        return PXR_ERR_INVALID_ARG;
    }
    const uint8_t* frames = d_frames + (size_t)e0 * c->cc.S * c->cc.H * c->cc.W * 3;
    uint16_t* out = d_out + (size_t)e0 * c->cc.Ho * c->cc.Wo * 32;
    if ((reinterpret_cast<uintptr_t>(frames) & 3u) || (reinterpret_cast<uintptr_t>(out) & 15u)) {
        err = "frames must be 4-byte and the output 16-byte aligned";
        return PXR_ERR_INVALID_ARG;
    }
    return pxr::launch_conv(c->cc, frames, n, out, c->n_groups, stream, err);
}

extern "C" {

int pxr_conv_create(const pxr_conv_desc* d, pxr_conv** out) {
    using pxr::set_error;
    if (!d || !out || !d->weights || !d->bias) return set_error(PXR_ERR_INVALID_ARG, "pxr_conv_create: null argument");
    if (d->kernel != 3 || d->stride != 2 || d->c_out != 32)
        return set_error(PXR_ERR_UNSUPPORTED, "pxr_conv_create: only kernel 3, stride 2, 32 output channels are built");
    if (d->n_stack < 1 || d->n_stack > 4) return set_error(PXR_ERR_UNSUPPORTED, "pxr_conv_create: n_stack must lie in [1,4]");
    if (d->in_h < 3 || d->in_h > 512 || d->in_w < 4 || d->in_w > 256 || (d->in_w & 3u))
        return set_error(PXR_ERR_UNSUPPORTED, "pxr_conv_create: height in [3,512], width in [4,256] and a multiple of 4");
    const uint32_t S = d->n_stack, cin = 3 * S;
    for (uint32_t i = 0; i < 9 * cin * 32; ++i)
        if (!std::isfinite(d->weights[i])) return set_error(PXR_ERR_INVALID_ARG, "pxr_conv_create: non-finite weight");
    for (uint32_t i = 0; i < 32; ++i)
        if (!std::isfinite(d->bias[i])) return set_error(PXR_ERR_INVALID_ARG, "pxr_conv_create: non-finite bias");

    pxr_conv* c = new (std::nothrow) pxr_conv();
    if (!c) return set_error(PXR_ERR_OOM, "pxr_conv_create: host allocation failed");
    pxr::ConvConsts& cc = c->cc;
    cc.H = d->in_h;
    cc.W = d->in_w;
    cc.S = S;
    cc.Ho = (cc.H - 3) / 2 + 1;
    cc.Wo = (cc.W - 3) / 2 + 1;
    cc.tiles_x = (cc.Wo + 31) / 32;
    cc.tiles_magic = (65536u + cc.tiles_x - 1) / cc.tiles_x;
    cc.relu = d->relu ? 1u : 0u;
    // band height: about 40 KB of LDS per workgroup so that four of them share a compute unit
    uint32_t band = 1;
    // (and the band's input must fit the registers that prefetch it)
    while (band < cc.Ho && S * (2 * (band + 1) + 1) * cc.W * 8u + 8192u <= 40u * 1024u &&
           S * (2 * (band + 1) + 1) * (cc.W / 4u) <= pxr::conv_max_quads())
        ++band;
    plan(c, band);
    if (pxr::conv_lds_bytes(cc) > 160u * 1024u || S * cc.rows_in * (cc.W / 4u) > pxr::conv_max_quads()) {
        delete c;
        return set_error(PXR_ERR_UNSUPPORTED, "pxr_conv_create: one output row of this input does not fit a workgroup");
    }

    // A operands: for instruction j = s*3 + ky, lane (g = lane/32, m = lane%32) holds matrix row m,
    // k = 8g..8g+7 = (pixel offset 2g + t/4, channel t%4); row 8a + 4h + b is output channel 16h + 4a + b.
    std::vector<uint16_t> wtab((size_t)3 * S * 64 * 8, 0);
    for (uint32_t s = 0; s < S; ++s)
        for (uint32_t ky = 0; ky < 3; ++ky)
            for (uint32_t lane = 0; lane < 64; ++lane) {
                const uint32_t g = lane >> 5, m = lane & 31u;
                const uint32_t co = 16 * ((m >> 2) & 1u) + 4 * (m >> 3) + (m & 3u);
                for (uint32_t t = 0; t < 8; ++t) {
                    const uint32_t kx = 2 * g + t / 4, ch = t % 4;
                    if (kx > 2 || ch > 2) continue;
                    wtab[(((size_t)(s * 3 + ky)) * 64 + lane) * 8 + t] =
                        bf16_rne(d->weights[((ky * 3 + kx) * cin + 3 * s + ch) * 32 + co]);
                }
            }
    const size_t wbytes = wtab.size() * 2, total = wbytes + 32 * 4;
    std::vector<unsigned char> staging(total);
    std::memcpy(staging.data(), wtab.data(), wbytes);
    std::memcpy(staging.data() + wbytes, d->bias, 32 * 4);
    hipError_t hrc = hipMalloc(&c->d_tables, total);
    if (hrc != hipSuccess) {
        delete c;
        return set_error(hrc == hipErrorOutOfMemory ? PXR_ERR_OOM : PXR_ERR_DEVICE,
                         std::string("pxr_conv_create: hipMalloc failed: ") + hipGetErrorString(hrc));
    }
    hrc = hipMemcpy(c->d_tables, staging.data(), total, hipMemcpyHostToDevice);
    int dev = 0;
    hipDeviceProp_t prop;
    if (hrc == hipSuccess) hrc = hipGetDevice(&dev);
    if (hrc == hipSuccess) hrc = hipGetDeviceProperties(&prop, dev);
    std::string err;
    if (hrc != hipSuccess || pxr::prepare_conv_kernels(err) != PXR_OK) {
        (void)hipFree(c->d_tables);
        delete c;
        return set_error(PXR_ERR_DEVICE, "pxr_conv_create: " + (hrc != hipSuccess ? std::string(hipGetErrorString(hrc)) : err));
    }
    cc.wtab = static_cast<const uint32_t*>(c->d_tables);
    cc.bias = reinterpret_cast<const float*>(static_cast<const unsigned char*>(c->d_tables) + wbytes);
    c->n_cus = (uint32_t)prop.multiProcessorCount;
    c->default_band = cc.band_rows;
    const uint32_t per_cu = std::max(1u, std::min(8u, (160u * 1024u) / pxr::conv_lds_bytes(cc)));
    c->default_groups = c->n_groups = c->n_cus * per_cu;
    *out = c;
    return PXR_OK;
}

int pxr_conv_destroy(pxr_conv* c) {
    if (!c) return PXR_OK;
    const hipError_t hrc = hipFree(c->d_tables);
    delete c;
    if (hrc != hipSuccess) return pxr::set_error(PXR_ERR_DEVICE, std::string("pxr_conv_destroy: hipFree failed: ") + hipGetErrorString(hrc));
    return PXR_OK;
}

int pxr_conv_info(const pxr_conv* c, uint32_t* out_h, uint32_t* out_w, uint32_t* band_rows, uint32_t* lds_bytes,
                  uint32_t* n_groups) {
    if (!c) return pxr::set_error(PXR_ERR_INVALID_ARG, "pxr_conv_info: null handle");
    if (out_h) *out_h = c->cc.Ho;
    if (out_w) *out_w = c->cc.Wo;
    if (band_rows) *band_rows = c->cc.band_rows;
    if (lds_bytes) *lds_bytes = pxr::conv_lds_bytes(c->cc);
    if (n_groups) *n_groups = c->n_groups;
    return PXR_OK;
}

int pxr_conv_set_tuning(pxr_conv* c, uint32_t band_rows, uint32_t n_groups) {
    if (!c) return pxr::set_error(PXR_ERR_INVALID_ARG, "pxr_conv_set_tuning: null handle");
    const pxr::ConvConsts saved = c->cc;
    plan(c, band_rows ? std::min(band_rows, c->cc.Ho) : c->default_band);
    if (pxr::conv_lds_bytes(c->cc) > 160u * 1024u || c->cc.S * c->cc.rows_in * (c->cc.W / 4u) > pxr::conv_max_quads()) {
        c->cc = saved;
        return pxr::set_error(PXR_ERR_UNSUPPORTED, "pxr_conv_set_tuning: band does not fit a workgroup");
    }
    c->n_groups = n_groups ? n_groups : c->default_groups;
    return PXR_OK;
}

int pxr_conv_forward(pxr_conv* c, const uint8_t* d_frames, uint32_t B, uint16_t* d_out, void* hip_stream) {
    using pxr::set_error;
    if (!c || !d_frames || !d_out) return set_error(PXR_ERR_INVALID_ARG, "pxr_conv_forward: null argument");
    std::string err;
    const int rc = pxr::conv_envs(c, d_frames, 0, B, d_out, hip_stream, err);
    if (rc != PXR_OK) return set_error(rc, "pxr_conv_forward: " + err);
    return PXR_OK;
}

}  // extern "C"
