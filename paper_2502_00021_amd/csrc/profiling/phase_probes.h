// PROFILING BUILDS ONLY: never included by the library's own build (render.hip includes it under
// -DPXR_PROFILING_BUILD, which only `build.py --define ... --out FILE` sets).  Defines the render kernel's phase
// probes in one of two forms:
//   -DPXR_PHASE_TIMING   the first wavefront of every workgroup notes the shader clock at each phase boundary
//                        (add -DPXR_WAVE_ARRIVAL for every wavefront's arrival at every barrier)
//   -DPXR_STOP_AFTER=k   the kernel returns after phase k (hardware-counter deltas give per-phase cost);
//                        the frames are NOT rendered
#ifndef PXR_PHASE_PROBES_H
#define PXR_PHASE_PROBES_H

#if defined(PXR_PHASE_TIMING)
// The first wavefront of every workgroup notes the clock at each phase boundary (in
// registers) and lane 0 adds the spans to global counters when the kernel ends (1024 sets of counters: one
// shared set would serialise the kernel's tail).
__device__ unsigned long long g_phase_cycles[1024 * 8];
__device__ unsigned long long g_wave_arrival[1024 * 8 * 16];  // per barrier and wavefront: arrival after the barrier's first wavefront
#define PXR_PHASE_BEGIN()                      \
    unsigned long long phase_span[8] = {0};    \
    unsigned long long phase_t0 = __builtin_readcyclecounter()
#define PXR_PHASE_MARK(i)                                                \
    {                                                                    \
        const unsigned long long now = __builtin_readcyclecounter();    \
        phase_span[i] += now - phase_t0;                                 \
        phase_t0 = now;                                                  \
    }
// (with -DPXR_WAVE_ARRIVAL: a barrier that also notes, per wavefront, how long after the first one it arrived;
// the second barrier it needs slows the kernel, so the phase clocks are best read without it)
#ifndef PXR_WAVE_ARRIVAL
#define PXR_TIMED_BARRIER(i) __syncthreads()
#else
#define PXR_TIMED_BARRIER(i)                                                                              \
    {                                                                                                         \
        unsigned long long* arr = reinterpret_cast<unsigned long long*>(lds + sc.lds_misc + 128);             \
        if (lane == 0) arr[tid >> 6] = __builtin_readcyclecounter();                                          \
        __syncthreads();                                                                                      \
        if (tid < NT / 64) {                                                                                  \
            unsigned long long first = arr[0];                                                                \
            for (uint32_t k = 1; k < NT / 64; ++k) first = arr[k] < first ? arr[k] : first;                   \
            atomicAdd(&g_wave_arrival[((blockIdx.x & 1023u) * 8u + (i)) * 16u + tid], arr[tid] - first);      \
        }                                                                                                     \
        __syncthreads();                                                                                      \
    }
#endif
#define PXR_PHASE_END()                                                                                      \
    if (tid == 0) {                                                                                          \
        for (int i = 0; i < 7; ++i) atomicAdd(&g_phase_cycles[(blockIdx.x & 1023u) * 8u + i], phase_span[i]); \
    }
#elif defined(PXR_STOP_AFTER)
// The kernel ends after phase PXR_STOP_AFTER (counter deltas give per-phase cost).
#define PXR_PHASE_BEGIN()
#define PXR_PHASE_MARK(i) \
    if ((i) == PXR_STOP_AFTER) return
#define PXR_TIMED_BARRIER(i) __syncthreads()
#define PXR_PHASE_END()
#else
#error "a profiling build defines PXR_PHASE_TIMING or PXR_STOP_AFTER"
#endif

#endif
