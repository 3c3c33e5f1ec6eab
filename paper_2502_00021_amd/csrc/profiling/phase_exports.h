// PROFILING BUILDS ONLY (see phase_probes.h): host-side readers of the phase clocks, exported beside the C ABI.
// Included inside render.hip's anonymous namespace, after the kernel.
extern "C" int pxr_debug_wave_arrival(unsigned long long* out) {  // out[8][16]
    static unsigned long long host[1024 * 8 * 16];
    if (hipMemcpyFromSymbol(host, HIP_SYMBOL(g_wave_arrival), sizeof(host)) != hipSuccess) return 1;
    for (int i = 0; i < 128; ++i) out[i] = 0;
    for (int k = 0; k < 1024; ++k)
        for (int i = 0; i < 128; ++i) out[i] += host[k * 128 + i];
    for (auto& h : host) h = 0;
    return hipMemcpyToSymbol(HIP_SYMBOL(g_wave_arrival), host, sizeof(host)) != hipSuccess;
}

extern "C" int pxr_debug_phase_cycles(unsigned long long* out, int reset) {
    static unsigned long long host[1024 * 8];
    if (out) {
        if (hipMemcpyFromSymbol(host, HIP_SYMBOL(g_phase_cycles), sizeof(host)) != hipSuccess) return 1;
        for (int i = 0; i < 8; ++i) out[i] = 0;
        for (int k = 0; k < 1024; ++k)
            for (int i = 0; i < 8; ++i) out[i] += host[k * 8 + i];
    }
    if (reset) {
        for (auto& h : host) h = 0;
        if (hipMemcpyToSymbol(HIP_SYMBOL(g_phase_cycles), host, sizeof(host)) != hipSuccess) return 1;
    }
    return 0;
}
