// The reverse sweep of a repeated Apply for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops): the checkpoints that dol_iterate_backward_ckpt takes through a workspace argument
// live in a file-scope device array here.  The call replays the forward sweep into that array (a checkpoint every
// kEvery rounds) and then walks the rounds backwards from it, with the kernels of the checkpointed entry points.
#include "internal.h"

#include <mutex>

using namespace dol;

namespace {

constexpr int32_t kEvery = 8;                          // checkpoint interval
constexpr size_t kScratchFloats = size_t(4) << 20;     // 16 MiB per device, held until the process ends

// One copy per device.  Host code never uses this name as an address: the address on the current device comes from
// hipGetSymbolAddress (scratch_address) and is what the launches receive.
static __device__ __align__(256) float scratch[kScratchFloats];

dol_status scratch_address(float **ptr)
{
    static std::mutex mu;
    static float *addr[64] = {};
    int dev = 0;
    DOL_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(DOL_EUNSUPPORTED, "device index %d outside 0..63", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        float *p = nullptr;
        DOL_HIP(hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)));
        if (!p) return fail(DOL_EHIP, "hipGetSymbolAddress returned no address for the built-in workspace");
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return DOL_OK;
}

}  // namespace

extern "C" dol_status dol_iterate_backward_noalloc(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f,
                                                   int32_t rounds, const float *grad_out, int64_t grad_out_ld,
                                                   float *grad_r0, float *grad_e, void *hip_stream)
{
    if (dol_status st = check_iterate(e, f, rounds)) return st;
    if (dol_status st = check_r0(r0, e, f)) return st;
    if (e->batch == 0 || f->na == 0 || (!grad_r0 && !grad_e)) return DOL_OK;
    if (!grad_out) return fail(DOL_EINVAL, "grad_out is NULL");
    if (grad_out_ld < f->na) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(grad_out_ld), f->na);
    const int32_t every = std::max<int32_t>(1, std::min<int32_t>(kEvery, std::max<int32_t>(rounds, 1)));
    const int32_t n_ckpt = dol_iterate_ckpt_count(rounds, every);
    const int64_t need = static_cast<int64_t>(n_ckpt) * e->batch * f->na;
    if (need > static_cast<int64_t>(kScratchFloats))
        return fail(DOL_EUNSUPPORTED, "%d checkpoints of %d x %d tags are %lld floats, the built-in workspace holds %zu",
                    n_ckpt, e->batch, f->na, static_cast<long long>(need), kScratchFloats);
    float *ws = nullptr;
    if (dol_status st = scratch_address(&ws)) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // every checkpoint the reverse sweep reads is written by the forward sweep of this same call: nothing to clear
    if (dol_status st = launch_iterate_fwd(r0, e, f, rounds, nullptr, ws, every, nullptr, 0, stream)) return st;
    return launch_iterate_bwd(e, f, rounds, nullptr, r0->prob, r0->ld, ws, every, grad_out, grad_out_ld, grad_r0, grad_e, stream);
}
