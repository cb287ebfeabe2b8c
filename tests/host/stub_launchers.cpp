// Stand-ins for the kernel launchers so that the host-side argument checks of the C ABI can be
// built with plain g++ and run under AddressSanitizer / UBSan without a GPU: they record that a
// launch was requested and touch none of the (fake) device pointers.
#include "internal.h"

namespace mics {
int g_launches = 0;
int launch_reorder(void*, const PtrTable&, size_t, size_t, int, int, bool, void*) { ++g_launches; return 0; }
int launch_reduce_scatter_accum(float*, const PtrTable&, size_t, int, bool, int, void*) { ++g_launches; return 0; }
int launch_replica_average(float*, const PtrTable&, size_t, int, float, void*) { ++g_launches; return 0; }
int launch_adam(float*, float*, float*, uint16_t*, bool, const float*, size_t, const AdamScalars&, void*) { ++g_launches; return 0; }
int launch_avg_adam(float*, float*, float*, uint16_t*, bool, const PtrTable&, int, float, size_t, const AdamScalars&, void*) { ++g_launches; return 0; }
// the real launchers issue one kernel launch per kMaxSegPerLaunch segments
int launch_reorder_coalesced(void*, const PtrTable&, const Segment*, int n, int, int, int, bool, void*)
{
    g_launches += (n + kMaxSegPerLaunch - 1) / kMaxSegPerLaunch;
    return 0;
}
int launch_reduce_coalesced(float*, const PtrTable&, const Segment*, int n, int, bool, int, void*)
{
    g_launches += (n + kMaxSegPerLaunch - 1) / kMaxSegPerLaunch;
    return 0;
}
void set_blocks_per_cu(int) {}
void set_stream_threshold_bytes(size_t) {}
void set_launch_shape(int, int, int) {}
const char* hip_error_text(int) { return "stub"; }
}  // namespace mics
