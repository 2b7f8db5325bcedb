// Host-only stand-ins for the device side of libatb (the HIP translation units), so that the C ABI's
// argument handling (atb_api.cpp) and the model / selector (atb_model.cpp) can be linked into a plain
// host program and run under AddressSanitizer + UndefinedBehaviorSanitizer.  Every launch "fails" with
// hipErrorNoDevice, which is also what the real library reports on a machine without a GPU.
#include "atb_internal.h"

namespace atb {
namespace {
hipError_t no_device(const GemmParams &, hipStream_t) { return hipErrorNoDevice; }
hipError_t no_device_fmt(const GemmParams &, int, int, hipStream_t) { return hipErrorNoDevice; }

Instance make(int T_MA, int T_MC, int T_K, int T_N, int wm, int wn, int lds, bool fmt)
{
    Instance i{};
    i.T_MA = T_MA; i.T_MC = T_MC; i.T_K = T_K; i.T_N = T_N;
    i.wave_m = wm; i.wave_n = wn; i.threads = wm * wn * 64; i.lds_bytes = lds;
    i.wg_per_cu = 160 * 1024 / lds;
    i.mfma_rows = (wm * wn == 8) ? 16 : 32;
    i.eff_scale = 1.0; i.lone_cap = 0.0;
    i.launch = &no_device;
    i.launch_fmt = fmt ? &no_device_fmt : nullptr;
    i.has_b_transposed = fmt && T_K == 64 && T_MC * T_N >= 128 * 256;
    return i;
}
const Instance g_table[] = {
    make(256, 256, 64, 256, 2, 4, 139264, true), make(128, 256, 64, 256, 2, 4, 102400, true),
    make(32, 256, 128, 256, 1, 4, 148480, false), make(32, 64, 64, 64, 1, 2, 25600, true),
};
}  // namespace

int instance_count() { return (int)(sizeof g_table / sizeof g_table[0]); }
const Instance &instance(int i) { return g_table[i]; }
int find_instance(int T_MA, int T_MC, int T_K, int T_N)
{
    for (int i = 0; i < instance_count(); ++i)
        if (g_table[i].T_MA == T_MA && g_table[i].T_MC == T_MC && g_table[i].T_K == T_K && g_table[i].T_N == T_N) return i;
    return -1;
}
hipError_t launch_quantize(const float *, int64_t, int8_t *, uint8_t *, int64_t, int64_t, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_decode(const int8_t *, const uint8_t *, uint16_t *, int64_t, int64_t, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_mfma_probe(float *, unsigned long long *, int, int, int, int, hipStream_t) { return hipErrorNoDevice; }
double mfma_probe_flop(int workgroups, int iters) { return 8.0 * workgroups * iters * 32.0 * 32768.0; }
size_t mfma_probe_sink_bytes(int workgroups) { return (size_t)workgroups * 512 * 4; }
}  // namespace atb
