// leap_project_host / leap_backproject_host: the projector pair on arrays in HOST memory ("Core CUDA Implementation":
// the library accepts data on the CPU as well as on the GPU and moves it itself; "Performance and Memory Usage" times
// the operators with and without that transfer).
//
// One call runs a three-stage pipeline over the items of the batch: item b+1 is uploaded while item b is projected
// and item b-1 is downloaded, on three streams of the default priority (two of them busy with copies) tied together
// by events.  Pageable host memory goes through pinned staging buffers in chunks, two per direction, so that the
// CPU's copy of one chunk overlaps the DMA of the previous one; memory the runtime reports as pinned is handed to the
// DMA engines directly.  The device arrays (two inputs, two outputs), the pinned buffers, streams and events belong to
// the handle, are created by its first host call and freed with it.
#include <algorithm>
#include <cstring>
#include <thread>

#include "leap_internal.h"

namespace {

constexpr int COPY_THREADS = 4;                     // CPU threads sharing one chunk's copy to / from pinned memory

void parallel_copy(void *dst, const void *src, size_t bytes)
{
    if (bytes < ((size_t)1 << 20)) {                // not worth a thread
        std::memcpy(dst, src, bytes);
        return;
    }
    const size_t part = ((bytes / COPY_THREADS) + 4095) & ~(size_t)4095;
    std::thread helpers[COPY_THREADS - 1];
    int started = 0;
    size_t handed = std::min(part, bytes);          // the calling thread copies [0, part) itself
    for (int t = 1; t < COPY_THREADS && handed < bytes; ++t) {
        const size_t off = handed, len = std::min(part, bytes - off);
        try {
            helpers[started] = std::thread([=] { std::memcpy((char *)dst + off, (const char *)src + off, len); });
        } catch (...) {
            break;                                  // no thread to be had: the caller copies the rest below
        }
        ++started;
        handed += len;
    }
    std::memcpy(dst, src, std::min(part, bytes));
    if (handed < bytes) std::memcpy((char *)dst + handed, (const char *)src + handed, bytes - handed);
    for (int t = 0; t < started; ++t) helpers[t].join();
}

bool is_pinned(const void *p)
{
    hipPointerAttribute_t attr;
    std::memset(&attr, 0, sizeof attr);
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();            // an ordinary pointer is reported as an error: clear it
        return false;
    }
    return attr.type == hipMemoryTypeHost;
}

}  // namespace

struct LeapHostStage {
    hipStream_t s_up = nullptr, s_run = nullptr, s_down = nullptr;
    float *d_in[2] = {nullptr, nullptr}, *d_out[2] = {nullptr, nullptr};
    size_t in_floats = 0, out_floats = 0;           // capacity of each device array
    char *pin_up[2] = {nullptr, nullptr}, *pin_down[2] = {nullptr, nullptr};   // G->stage_chunk bytes each
    hipEvent_t up_slot[2] = {nullptr, nullptr}, down_slot[2] = {nullptr, nullptr};     // last DMA of a staging buffer
    hipEvent_t uploaded[2] = {nullptr, nullptr}, ran[2] = {nullptr, nullptr}, downloaded[2] = {nullptr, nullptr};
};

void leap_host_stage_free(leap_geometry *G)
{
    LeapHostStage *H = G->host_stage;
    if (!H) return;
    for (int q = 0; q < 2; ++q) {
        if (H->d_in[q]) (void)hipFree(H->d_in[q]);
        if (H->d_out[q]) (void)hipFree(H->d_out[q]);
        if (H->pin_up[q]) (void)hipHostFree(H->pin_up[q]);
        if (H->pin_down[q]) (void)hipHostFree(H->pin_down[q]);
        for (hipEvent_t e : {H->up_slot[q], H->down_slot[q], H->uploaded[q], H->ran[q], H->downloaded[q]})
            if (e) (void)hipEventDestroy(e);
    }
    for (hipStream_t s : {H->s_up, H->s_run, H->s_down})
        if (s) (void)hipStreamDestroy(s);
    delete H;
    G->host_stage = nullptr;
}

static int stage_create(LeapHostStage *H)
{
    LEAP_HIP_CHECK(hipStreamCreateWithFlags(&H->s_up, hipStreamNonBlocking));
    LEAP_HIP_CHECK(hipStreamCreateWithFlags(&H->s_run, hipStreamNonBlocking));
    LEAP_HIP_CHECK(hipStreamCreateWithFlags(&H->s_down, hipStreamNonBlocking));
    for (int q = 0; q < 2; ++q)
        for (hipEvent_t *e : {&H->up_slot[q], &H->down_slot[q], &H->uploaded[q], &H->ran[q], &H->downloaded[q]})
            LEAP_HIP_CHECK(hipEventCreateWithFlags(e, hipEventDisableTiming));
    return LEAP_OK;
}

static int stage_prepare(const leap_geometry *G, size_t in_floats, size_t out_floats, int slots)
{
    if (!G->host_stage) {
        LeapHostStage *H = new (std::nothrow) LeapHostStage;
        if (!H) {
            leap_set_error("out of host memory");
            return LEAP_INVALID_ARG;
        }
        G->host_stage = H;
        const int rc = stage_create(H);
        if (rc != LEAP_OK) {                        // no half-built stage is kept for the next call to trip over
            leap_host_stage_free(const_cast<leap_geometry *>(G));
            return rc;
        }
    }
    LeapHostStage *H = G->host_stage;
    for (int q = 0; q < 2; ++q) {
        if (!H->pin_up[q]) LEAP_HIP_CHECK(hipHostMalloc((void **)&H->pin_up[q], G->stage_chunk, hipHostMallocDefault));
        if (!H->pin_down[q]) LEAP_HIP_CHECK(hipHostMalloc((void **)&H->pin_down[q], G->stage_chunk, hipHostMallocDefault));
    }
    // the same handle serves both directions: the arrays grow to the larger of volume and sinogram when needed
    if (H->in_floats < in_floats || H->out_floats < out_floats) {
        for (int q = 0; q < 2; ++q) {
            if (H->d_in[q]) (void)hipFree(H->d_in[q]);
            if (H->d_out[q]) (void)hipFree(H->d_out[q]);
            H->d_in[q] = H->d_out[q] = nullptr;
        }
        H->in_floats = H->out_floats = 0;
    }
    for (int q = 0; q < slots; ++q) {
        if (!H->d_in[q]) LEAP_HIP_CHECK(hipMalloc((void **)&H->d_in[q], std::max(in_floats, H->in_floats) * sizeof(float)));
        if (!H->d_out[q]) LEAP_HIP_CHECK(hipMalloc((void **)&H->d_out[q], std::max(out_floats, H->out_floats) * sizeof(float)));
    }
    H->in_floats = std::max(in_floats, H->in_floats);
    H->out_floats = std::max(out_floats, H->out_floats);
    return LEAP_OK;
}

namespace {

// One direction of one item, cut into chunks; `step` moves the next chunk, if one is left (moved = true).
struct Transfer {
    LeapHostStage *H = nullptr;
    bool up = false, pinned = false, active = false;
    char *host = nullptr;
    char *dev = nullptr;
    size_t bytes = 0, next = 0, chunk = 0;
    int slot = 0;
    // download only: chunks whose DMA was issued and whose copy out of the staging buffer is still owed
    char *owed_dst[2] = {nullptr, nullptr};
    size_t owed_len[2] = {0, 0};

    int drain(int q)
    {
        if (!owed_dst[q]) return LEAP_OK;
        LEAP_HIP_CHECK(hipEventSynchronize(H->down_slot[q]));
        parallel_copy(owed_dst[q], H->pin_down[q], owed_len[q]);
        owed_dst[q] = nullptr;
        return LEAP_OK;
    }

    int step(bool &moved)
    {
        moved = false;
        if (!active || next >= bytes) return LEAP_OK;
        const size_t len = std::min(chunk, bytes - next);
        if (up) {
            if (pinned) {
                LEAP_HIP_CHECK(hipMemcpyAsync(dev + next, host + next, len, hipMemcpyHostToDevice, H->s_up));
            } else {
                LEAP_HIP_CHECK(hipEventSynchronize(H->up_slot[slot]));      // the buffer's previous DMA has read it
                parallel_copy(H->pin_up[slot], host + next, len);
                LEAP_HIP_CHECK(hipMemcpyAsync(dev + next, H->pin_up[slot], len, hipMemcpyHostToDevice, H->s_up));
                LEAP_HIP_CHECK(hipEventRecord(H->up_slot[slot], H->s_up));
            }
        } else {
            if (pinned) {
                LEAP_HIP_CHECK(hipMemcpyAsync(host + next, dev + next, len, hipMemcpyDeviceToHost, H->s_down));
            } else {
                const int rc = drain(slot);
                if (rc != LEAP_OK) return rc;
                LEAP_HIP_CHECK(hipMemcpyAsync(H->pin_down[slot], dev + next, len, hipMemcpyDeviceToHost, H->s_down));
                LEAP_HIP_CHECK(hipEventRecord(H->down_slot[slot], H->s_down));
                owed_dst[slot] = host + next;
                owed_len[slot] = len;
            }
        }
        slot ^= 1;
        next += len;
        moved = true;
        return LEAP_OK;
    }

    int finish()
    {
        for (int q = 0; q < 2; ++q) {
            const int rc = drain(q);
            if (rc != LEAP_OK) return rc;
        }
        active = false;
        return LEAP_OK;
    }
};

// The steps of the pipeline; returns at the first failure with work possibly still in flight on the three streams.
int pipeline_steps(const leap_geometry *G, LeapHostStage *H, const float *h_in, float *h_out, size_t nin, size_t nout,
                   int batch, bool forward)
{
    const bool in_pinned = is_pinned(h_in), out_pinned = is_pinned(h_out);
    int rc = LEAP_OK;
    // step s: upload item s, run item s-1, download item s-2
    Transfer upload, download;
    upload.H = download.H = H;
    upload.chunk = download.chunk = G->stage_chunk;
    upload.up = true;
    for (int s = 0; s < batch + 2 && rc == LEAP_OK; ++s) {
        const int iu = s, ir = s - 1, id = s - 2;
        if (ir >= 0 && ir < batch) {
            const int q = ir & 1;
            LEAP_HIP_CHECK(hipStreamWaitEvent(H->s_run, H->uploaded[q], 0));
            if (ir >= 2) LEAP_HIP_CHECK(hipStreamWaitEvent(H->s_run, H->downloaded[q], 0));     // d_out[q] was read out
            rc = forward ? leap_launch_project_batch(G, H->d_in[q], H->d_out[q], 1, H->s_run)
                         : leap_launch_backproject_batch(G, H->d_in[q], H->d_out[q], 1, H->s_run);
            if (rc != LEAP_OK) break;
            LEAP_HIP_CHECK(hipEventRecord(H->ran[q], H->s_run));
        }
        if (iu < batch) {
            const int q = iu & 1;
            if (iu >= 2) LEAP_HIP_CHECK(hipStreamWaitEvent(H->s_up, H->ran[q], 0));             // d_in[q] was consumed
            upload.active = true; upload.pinned = in_pinned;
            upload.host = (char *)const_cast<float *>(h_in + (size_t)iu * nin);
            upload.dev = (char *)H->d_in[q];
            upload.bytes = nin * sizeof(float); upload.next = 0;
        }
        if (id >= 0 && id < batch) {
            const int q = id & 1;
            LEAP_HIP_CHECK(hipStreamWaitEvent(H->s_down, H->ran[q], 0));
            download.active = true; download.pinned = out_pinned;
            download.host = (char *)(h_out + (size_t)id * nout);
            download.dev = (char *)H->d_out[q];
            download.bytes = nout * sizeof(float); download.next = 0;
        }
        // the chunks of the two transfers of this step, alternating
        for (bool more = true; more && rc == LEAP_OK;) {
            bool a = false, b = false;
            rc = upload.step(a);
            if (rc == LEAP_OK) rc = download.step(b);
            more = a || b;
        }
        if (rc != LEAP_OK) break;
        if (upload.active) {
            LEAP_HIP_CHECK(hipEventRecord(H->uploaded[iu & 1], H->s_up));
            upload.active = false;
        }
        if (download.active) {
            LEAP_HIP_CHECK(hipEventRecord(H->downloaded[id & 1], H->s_down));
            rc = download.finish();
        }
    }
    return rc;
}

int run_host_pipeline(const leap_geometry *G, const float *h_in, float *h_out, int batch, bool forward)
{
    const SfGeom &g = G->g;
    const size_t nvol = (size_t)g.nx * g.ny * g.nz, nsino = (size_t)g.nviews * g.nrows * g.ncols;
    const size_t nin = forward ? nvol : nsino, nout = forward ? nsino : nvol;
    int device = -1;
    LEAP_HIP_CHECK(hipGetDevice(&device));
    if (device != G->device) {
        leap_set_error("the handle was created on another device than the current one");
        return LEAP_INVALID_ARG;
    }
    std::lock_guard<std::mutex> lock(G->host_mutex);
    int rc = stage_prepare(G, nin, nout, batch > 1 ? 2 : 1);
    if (rc != LEAP_OK) return rc;
    LeapHostStage *H = G->host_stage;
    rc = pipeline_steps(G, H, h_in, h_out, nin, nout, batch, forward);
    // the call returns with the outputs in place; after a failure the streams are still drained before the buffers
    // can be touched again
    const hipError_t e1 = hipStreamSynchronize(H->s_up), e2 = hipStreamSynchronize(H->s_run), e3 = hipStreamSynchronize(H->s_down);
    if (rc != LEAP_OK) return rc;
    LEAP_HIP_CHECK(e1);
    LEAP_HIP_CHECK(e2);
    LEAP_HIP_CHECK(e3);
    return LEAP_OK;
}

int check_host_call(const leap_geometry *G, const void *in, const void *out, int32_t batch)
{
    if (!G || !in || !out) {
        leap_set_error("null handle or data pointer");
        return LEAP_INVALID_ARG;
    }
    if (batch <= 0) {
        leap_set_error("batch must be positive");
        return LEAP_INVALID_ARG;
    }
    if (in == out) {
        leap_set_error("input and output must not alias");
        return LEAP_INVALID_ARG;
    }
    return LEAP_OK;
}

}  // namespace

extern "C" int leap_project_host(const leap_geometry *G, const float *h_vol, float *h_sino, int32_t batch)
{
    const int rc = check_host_call(G, h_vol, h_sino, batch);
    return rc != LEAP_OK ? rc : run_host_pipeline(G, h_vol, h_sino, batch, true);
}

extern "C" int leap_backproject_host(const leap_geometry *G, const float *h_sino, float *h_vol, int32_t batch)
{
    const int rc = check_host_call(G, h_sino, h_vol, batch);
    return rc != LEAP_OK ? rc : run_host_pipeline(G, h_sino, h_vol, batch, false);
}
