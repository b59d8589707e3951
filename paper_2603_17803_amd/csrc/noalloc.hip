// Scoring + selection for callers that cannot allocate device memory (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): the same kernels as swarm_score_select, with every piece
// of scratch -- the fp32 scores and the winners of the sliced selection -- laid out in one file-scope device
// array of fixed size instead of the context's growing buffers.
#include <mutex>

#include "common.h"

namespace {

constexpr size_t SCRATCH_BYTES = SWARM_STATIC_SCRATCH_BYTES;
// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress: kernels and copies get the device address resolved below.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};     // device address of `scratch` on each device, resolved once

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

}  // namespace

swarm_status swarm_static_scratch_init(swarm_ctx* ctx) {
    if (ctx->device < 0 || ctx->device >= MAX_DEVICES) {
        snprintf(ctx->err, sizeof(ctx->err), "device %d is beyond the %d devices the static scratch is tracked for", ctx->device, MAX_DEVICES);
        return SWARM_EINVAL;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[ctx->device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));      // the current device's copy
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            snprintf(ctx->err, sizeof(ctx->err), "hipGetSymbolAddress of the static scratch failed: %s", hipGetErrorString(e));
            return SWARM_EHIP;
        }
        g_scratch_ptr[ctx->device] = ptr;
    }
    ctx->static_scratch = g_scratch_ptr[ctx->device];
    return SWARM_OK;
}

extern "C" swarm_status swarm_score_select_static(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t B, int32_t k,
                                                  int32_t* out_idx) {
    SWARM_ENTER(ctx);
    swarm_status st = swarm_check_score_args(ctx, "score_select_static", keys, q, B);
    if (st != SWARM_OK) return st;
    if (!out_idx) SWARM_REJECT(ctx, "score_select_static: NULL out_idx");
    if (k < 1 || k > keys->N) SWARM_REJECT(ctx, "score_select_static: k=%d outside [1,N=%d]", k, keys->N);
    if (!ctx->static_scratch) SWARM_REJECT(ctx, "score_select_static: the static scratch was not resolved for device %d", ctx->device);

    const int64_t rows = (int64_t)B * keys->H;
    const size_t scores_bytes = align256(sizeof(float) * (size_t)rows * keys->N);
    const size_t cand_bytes = align256(select_cand_bytes(rows, keys->N, k));
    const size_t need = scores_bytes + cand_bytes;
    if (need > SCRATCH_BYTES)
        SWARM_REJECT(ctx, "score_select_static: B=%d H=%d N=%d k=%d need %zu bytes of scratch, the static scratch holds %zu", B, keys->H,
                     keys->N, k, need, SCRATCH_BYTES);
    unsigned char* base = static_cast<unsigned char*>(ctx->static_scratch);
    float* scores = reinterpret_cast<float*>(base);
    const swarm_fixed_scratch fixed{reinterpret_cast<int32_t*>(base + scores_bytes), cand_bytes};
    // every byte a kernel reads from the scratch is written by an earlier kernel of this call: nothing to clear
    st = launch_score(ctx, keys, q, B, scores);
    if (st != SWARM_OK) return st;
    return launch_select(ctx, scores, rows, keys->N, k, out_idx, &fixed);
}
