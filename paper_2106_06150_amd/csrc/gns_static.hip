// gns_sample_blocks_static: gns_sample_blocks for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The per-batch scratch that a
// context otherwise keeps in the workspace the caller allocated -- device counters, the frontier mark
// bitmap, the batch hash map, row extents, hub list, sampler scratch, scan partials -- lives in one fixed
// array of the library instead.  The kernels are the ones gns_sample_blocks launches; they are handed the
// array's device address where they are otherwise handed the workspace.
#include <stdio.h>
#include "gns_internal.h"
#include <string.h>
#include "gns_kernels.hpp"

namespace gns {

constexpr size_t kStaticScratchBytes = (size_t) GNS_STATIC_SCRATCH_BYTES;

// One copy per GPU, held from the moment the library's code is loaded on that GPU until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress: the address that kernels and fills
// receive is the one that call returned with the device current.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];    // per device: address of that device's copy of `scratch`

// Called by gns_create with the context's device current.  Looks the array's address on this device up
// (once per device) and, if the per-batch scratch of this graph and config fits, makes the hidden context
// that gns_sample_blocks_static runs on.  All allocation (host mirror, events) happens here, none in the call.
gns_status static_scratch_setup(gns_ctx* root)
{
    root->static_child = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return ctx_fail(root, GNS_EHIP, "hipGetDevice", e);
    if (dev < 0 || dev >= kMaxDevices) return GNS_OK;             // no static path on such a device id
    if (!g_scratch_ptr[dev]) {
        // A failure here (the array could not be placed on this device) only disables
        // gns_sample_blocks_static, which then reports it; the context itself does not depend on the array.
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) {
            snprintf(root->static_err, sizeof(root->static_err), "static scratch array unavailable on device %d: %s", dev,
                     e != hipSuccess ? hipGetErrorString(e) : "null or misaligned device address");
            (void) hipGetLastError();
            return GNS_OK;
        }
        g_scratch_ptr[dev] = ptr;
    }
    if (root->lay.shared_begin > kStaticScratchBytes) return GNS_OK;   // too big: the entry point says so
    gns_ctx* child = nullptr;
    const gns_status st = make_child(root, g_scratch_ptr[dev], false, &child);   // eager launches, no capture
    if (st != GNS_OK) return st;
    root->static_child = child;
    return GNS_OK;
}

}  // namespace gns

using namespace gns;

extern "C" gns_status gns_sample_blocks_static(gns_ctx* ctx, uint64_t seed, const int32_t* seeds_dev, int32_t num_seeds,
                                               gns_block* blocks, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    gns_ctx* root = ctx->root;
    gns_ctx* c = root->static_child;
    if (!c && root->static_err[0]) {
        snprintf(ctx->err, sizeof(ctx->err), "gns_sample_blocks_static: %s", root->static_err);
        return GNS_EHIP;
    }
    if (!c) {
        snprintf(ctx->err, sizeof(ctx->err),
                 "gns_sample_blocks_static: the per-batch scratch of this graph and config needs %zu bytes, the "
                 "library's static array holds %zu", (size_t) root->lay.shared_begin, kStaticScratchBytes);
        return GNS_ECAPACITY;
    }
    gns_status st = check_batch_args(c, seeds_dev, num_seeds, blocks);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (st == GNS_OK) {
        const hipError_t er = before_cache_readers(c, s);
        if (er == hipErrorInvalidValue) st = ctx_fail(c, GNS_ESTATE, "more than 4 streams between two cache draws");
        else if (er != hipSuccess) st = ctx_fail(c, GNS_EHIP, "wait for the cache draw", er);
    }
    // The array keeps whatever the last call on this GPU left (possibly of another context with another
    // layout): everything that must start clean is cleared here, with fill kernels on the caller's stream.
    if (st == GNS_OK) {
        c->hash_parity = 0;
        c->batch_id = 0;
        c->bad_reported = 0;
        const hipError_t e = init_batch_scratch(c, s);
        if (e != hipSuccess) st = ctx_fail(c, GNS_EHIP, "static scratch init", e);
    }
    if (st == GNS_OK) {
        Group g;
        memset(&g, 0, sizeof(g));
        g.count = 1;
        g.ctx[0] = c;
        g.blocks[0] = blocks;
        BeginDyn dyn;
        fill_begin_dyn(g, &seed, &seeds_dev, &num_seeds, &dyn);
        st = enqueue_batch(g, dyn, s);
    }
    if (st == GNS_OK) {
        c->batch_id = 1;
        hipError_t e = hipMemcpyAsync(c->h_state, c->d_state, sizeof(DeviceState), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) st = ctx_fail(c, GNS_EHIP, "gns_sample_blocks_static wait", e);
    }
    if (st == GNS_OK) {
        for (int i = 0; i < c->config.num_layers; ++i) {
            blocks[i].num_dst = c->h_state->num_dst[i];
            blocks[i].num_src = c->h_state->num_dst[i + 1];
            blocks[i].num_edges = c->h_state->num_edges[i];
        }
        if (c->h_state->bad_seed != 0) st = ctx_fail(c, GNS_EINVAL, "seeds must be distinct node ids in [0, num_nodes)");
    }
    if (st != GNS_OK) snprintf(ctx->err, sizeof(ctx->err), "%s", c->err);
    return st;
}
