// ss_embbag_backward_update_noalloc: the update of ss_embbag_backward_update for
// callers that can neither allocate device memory nor bring a workspace (code
// under stream capture, serving loops, harnesses that forbid hipMalloc).  The
// sorted lookup lists, histograms and partial sums of the update live in a
// file-scope device array of fixed size instead of a caller's workspace; the
// kernels are the same, so the results are bit-identical.
//
// Each GPU holds its own copy of the array at its own address.  Host code never
// uses the array's name as an address: the name is a host-side stand-in.  The
// device address is looked up once per device with hipGetSymbolAddress, with
// that device current, and kept; kernels receive it as an ordinary argument.
#include <mutex>

#include "ss_common.h"

namespace {

static __device__ __align__(256) unsigned char scratch[SS_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on first use).
int32_t scratch_address(const char *who, void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return ss::fail(SS_ERR_HIP, "%s: no usable current device", who);
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return ss::fail(SS_ERR_HIP, "%s: hipGetSymbolAddress: %s", who,
                            hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SS_OK;
}

}  // namespace

using namespace ss;

extern "C" int32_t ss_embbag_backward_update_noalloc(const ss_tables *tables,
                                                     const int32_t *idx, int32_t Bcap,
                                                     int32_t L, const int32_t *n_valid,
                                                     const float *grad, float lr,
                                                     void *stream)
{
    const char *who = "ss_embbag_backward_update_noalloc";
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    if (Bcap < 1) return fail(SS_ERR_INVALID_ARG, "%s: batch = %d", who, Bcap);
    if (L < 1) return fail(SS_ERR_INVALID_ARG, "%s: L = %d", who, L);
    if ((int64_t)Bcap * L >= (1LL << 31) - 4096)
        return fail(SS_ERR_UNSUPPORTED, "%s: Bcap*L too large", who);
    if (!idx) return fail(SS_ERR_INVALID_ARG, "%s: idx is NULL", who);
    if (!grad) return fail(SS_ERR_INVALID_ARG, "%s: grad is NULL", who);
    if (reinterpret_cast<uintptr_t>(grad) % 16 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: grad is not 16-byte aligned", who);
    const size_t need = backward_ws_bytes(tables->num_tables, Bcap, L, tables->dim);
    if (need > (size_t)SS_NOALLOC_SCRATCH_BYTES)
        return fail(SS_ERR_WORKSPACE,
                    "%s: this shape needs %zu bytes of scratch, the built-in buffer has %zu "
                    "(use ss_embbag_backward_update with a workspace)",
                    who, need, (size_t)SS_NOALLOC_SCRATCH_BYTES);
    void *ws = nullptr;
    rc = scratch_address(who, &ws);
    if (rc) return rc;
    // no event pairs are created for these launches, whatever ss_profile_enable says
    ProfMute mute;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Every word of the scratch that a launch reads was written by an earlier launch
    // of the same call (lists, histograms, run states, partial sums): nothing has to
    // start at zero, and what the previous call left behind is never read.
    rc = launch_backward_prepare(tables, idx, Bcap, L, n_valid, ws, s);
    if (rc) return rc;
    return launch_backward_apply(tables, Bcap, L, grad, lr, ws, s);
}
