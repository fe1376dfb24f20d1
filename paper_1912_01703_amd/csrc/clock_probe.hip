// Measurement utility: the shader clock a GPU actually runs at while other kernels execute.
//
// One wave reads the shader-clock counter (s_memtime, which advances with the clock of the compute units)
// and the constant-rate counter (s_memrealtime) at its start, sleeps in short naps until the requested
// time has passed on the constant-rate counter, and reads both again.  The ratio of the two differences times the
// constant counter's rate is the average shader clock over that interval.  Launched on a second stream
// beside a benchmark's kernels it occupies one wave slot of one compute unit and issues no memory traffic
// until its two final stores.
#include "../../include/miconv.h"
#include "common.h"

namespace miconv {
namespace {

__global__ __launch_bounds__(64) void clock_sampler_kernel(unsigned long long* out, unsigned long long ticks, int max_naps) {
    const unsigned long long c0 = __builtin_readcyclecounter();
    const unsigned long long r0 = wall_clock64();
    unsigned long long r1 = r0;
    // ends when the time is up, and in any case after max_naps naps
    for (int nap = 0; nap < max_naps && r1 - r0 < ticks; ++nap) {
        __builtin_amdgcn_s_sleep(64);
        r1 = wall_clock64();
    }
    const unsigned long long c1 = __builtin_readcyclecounter();
    if (threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = r1 - r0;
    }
}

}  // namespace
}  // namespace miconv

extern "C" int miconv_sample_shader_clock(void* counts, unsigned duration_us, int* wall_clock_khz, void* hip_stream) {
    if (!counts || !wall_clock_khz) return MICONV_ERR_NULL;
    if (duration_us < 1 || duration_us > 1000000) return MICONV_ERR_SHAPE;
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0)
        return MICONV_ERR_LAUNCH;
    *wall_clock_khz = khz;
    const unsigned long long ticks = (unsigned long long)duration_us * (unsigned long long)khz / 1000ull;
    // a nap lasts 64 x 64 shader clocks (1.7 us at 2.4 GHz, longer at lower clocks): one nap per microsecond
    // asked for, plus a margin, is more than the duration needs and bounds the loop
    const int max_naps = (int)(duration_us) + 1024;
    miconv::clock_sampler_kernel<<<1, 64, 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<unsigned long long*>(counts), ticks, max_naps);
    return hipGetLastError() == hipSuccess ? MICONV_OK : MICONV_ERR_LAUNCH;
}
