// Context, status strings and the kernel-argument upload used by every entry point.
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include "px_internal.h"

px_status px_fail(px_ctx* ctx, px_status s, const char* fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof ctx->err, fmt, ap);
        va_end(ap);
    }
    return s;
}

px_status px_check_hip(px_ctx* ctx, hipError_t e, const char* what) {
    if (e == hipSuccess) return PX_OK;
    return px_fail(ctx, PX_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

// ------------------------------------------------------------------- upload
// Up to PX_UPLOAD_WORDS words travel inside the kernel arguments, so the copy is
// ordered with the stream, needs no pinned staging buffer and can be captured.
__global__ __launch_bounds__(256) void px_k_upload(uint64_t* __restrict__ dst, px_word_pack pack,
                                                   int n, uint32_t* __restrict__ zero, int nzero) {
    int t = threadIdx.x;
    if (t < n) dst[t] = pack.w[t];
    for (int i = t; i < nzero; i += blockDim.x) zero[i] = 0u;
}

px_status px_upload_words(px_ctx* ctx, uint64_t* dst, const uint64_t* host_words, int n,
                          uint32_t* zero, int nzero, hipStream_t stream) {
    int done = 0;
    do {
        px_word_pack pack;
        int m = n - done;
        if (m > PX_UPLOAD_WORDS) m = PX_UPLOAD_WORDS;
        if (m > 0) memcpy(pack.w, host_words + done, (size_t) m * sizeof(uint64_t));
        px_k_upload<<<1, 256, 0, stream>>>(dst + done, pack, m, done == 0 ? zero : nullptr,
                                           done == 0 ? nzero : 0);
        px_status s = px_check_hip(ctx, hipGetLastError(), "upload launch");
        if (s != PX_OK) return s;
        done += m;
    } while (done < n);
    return PX_OK;
}

// ------------------------------------------------------------------ context

extern "C" px_status px_create(px_ctx** out, int device) {
    if (!out) return PX_ERR_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count)
        return PX_ERR_DEVICE;
    px_ctx* ctx = (px_ctx*) calloc(1, sizeof(px_ctx));
    if (!ctx) return PX_ERR_DEVICE;
    ctx->device = device;
    ctx->wait_polls = PX_WAIT_POLLS_DEFAULT;
    int prev = 0;
    (void) hipGetDevice(&prev);
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) e = hipMalloc((void**) &ctx->d_words, PXW_TOTAL * sizeof(uint64_t));
    if (e == hipSuccess) e = hipMalloc((void**) &ctx->d_flags, 64 * sizeof(uint32_t));
    if (e == hipSuccess) e = hipHostMalloc((void**) &ctx->h_flags, 64 * sizeof(uint32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipMemset(ctx->d_flags, 0, 64 * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMalloc((void**) &ctx->d_part_pub, PX_PART_PUB_WORDS * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipMemset(ctx->d_part_pub, 0, PX_PART_PUB_WORDS * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess && px_partition_noalloc_setup(ctx) != PX_OK) e = hipErrorInvalidSymbol;
    (void) hipSetDevice(prev);
    if (e != hipSuccess) {
        px_destroy(ctx);
        return PX_ERR_DEVICE;
    }
    *out = ctx;
    return PX_OK;
}

extern "C" px_status px_destroy(px_ctx* ctx) {
    if (!ctx) return PX_OK;
    if (ctx->d_words) (void) hipFree(ctx->d_words);
    if (ctx->d_flags) (void) hipFree(ctx->d_flags);
    if (ctx->d_part_pub) (void) hipFree(ctx->d_part_pub);
    if (ctx->h_flags) (void) hipHostFree(ctx->h_flags);
    free(ctx);
    return PX_OK;
}

extern "C" px_status px_set_wait_limit(px_ctx* ctx, int64_t polls) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    if (polls < 0 || polls > (1ll << 30)) return px_fail(ctx, PX_ERR_INVALID_ARG, "wait limit %lld outside [0, 2^30]", (long long) polls);
    ctx->wait_polls = (int) polls;
    return PX_OK;
}

extern "C" const char* px_status_string(px_status s) {
    switch (s) {
        case PX_OK: return "ok";
        case PX_ERR_INVALID_ARG: return "invalid argument";
        case PX_ERR_INDEX_OUT_OF_RANGE: return "row id outside the table";
        case PX_ERR_SCRATCH_TOO_SMALL: return "scratch buffer too small";
        case PX_ERR_NOT_UNIQUE: return "row ids not distinct";
        case PX_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char* px_last_error(const px_ctx* ctx) { return ctx ? ctx->err : ""; }

__global__ void px_k_clear_flag(uint32_t* __restrict__ flags) {
    if (threadIdx.x == 0 && blockIdx.x == 0) flags[0] = 0u;
}

extern "C" px_status px_device_status(px_ctx* ctx, void* hip_stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t) hip_stream;
    ctx->h_flags[0] = 0u;
    px_status s = px_check_hip(ctx, hipMemcpyAsync(ctx->h_flags, ctx->d_flags, sizeof(uint32_t),
                                                   hipMemcpyDeviceToHost, stream), "status copy");
    if (s != PX_OK) return s;
    px_k_clear_flag<<<1, 64, 0, stream>>>(ctx->d_flags);
    s = px_check_hip(ctx, hipGetLastError(), "status launch");
    if (s != PX_OK) return s;
    s = px_check_hip(ctx, hipStreamSynchronize(stream), "status sync");
    if (s != PX_OK) return s;
    uint32_t f = ctx->h_flags[0];
    if (f & PXF_INTERNAL)
        return px_fail(ctx, PX_ERR_DEVICE, "a workgroup gave up waiting for another's head count: results of that call are invalid");
    if (f & PXF_BAD_ID)
        return px_fail(ctx, PX_ERR_INDEX_OUT_OF_RANGE, "a row id outside [0, vocab) reached the device");
    if (f & PXF_NOT_UNIQUE)
        return px_fail(ctx, PX_ERR_NOT_UNIQUE, "an update was handed the same row id twice in a row");
    return PX_OK;
}
