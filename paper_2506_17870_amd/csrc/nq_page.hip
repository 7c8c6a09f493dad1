// Switching between the full-bit and the part-bit model (paper Sec. 3.2.3 and Sec. 3.3):
// downgrading pages the lower-bit weights out, upgrading pages them in from storage.  On
// a GPU with a host master copy the page-out moves nothing; the page-in is one
// host-to-device copy that can overlap part-bit inference on another stream.
#include "nq_common.h"

using namespace nq;

extern "C" int nq_version(void) { return 1; }

extern "C" const char *nq_status_string(int status)
{
    switch (status) {
    case NQ_OK: return "ok";
    case NQ_ERR_INVALID_ARG: return "invalid argument";
    case NQ_ERR_UNSUPPORTED: return "unsupported nesting, format or layout";
    case NQ_ERR_SHAPE: return "inconsistent or too large shape";
    case NQ_ERR_ALIGN: return "page not 16-byte aligned";
    case NQ_ERR_NOT_RESIDENT: return "lower-bit page is paged out";
    case NQ_ERR_RANGE: return "buffer too small";
    case NQ_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

extern "C" nq_status nq_weight_init(nq_weight *w)
{
    if (!w) return NQ_ERR_INVALID_ARG;
    nq_status st = check_cfg(&w->cfg);
    if (st != NQ_OK) return st;
    if ((st = check_shape(w->N, w->K)) != NQ_OK) return st;
    const int h = w->cfg.n_bits - w->cfg.l_bits, l = low_field_bits(&w->cfg);
    if (w->high_bytes < nq_packed_bytes(w->N, w->K, h, w->cfg.layout)) return NQ_ERR_RANGE;
    if (w->low_bytes < nq_packed_bytes(w->N, w->K, l, w->cfg.layout)) return NQ_ERR_RANGE;
    if ((w->d_high && !aligned16(w->d_high)) || (w->d_low && !aligned16(w->d_low))) return NQ_ERR_ALIGN;
    hipEvent_t ev = nullptr;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    hipEvent_t ev2 = nullptr;
    if (hipEventCreateWithFlags(&ev2, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipEventDestroy(ev);
        return NQ_ERR_HIP;
    }
    w->low_event = ev;
    w->free_event = ev2;
    w->low_event_armed = 0;
    w->free_event_armed = 0;
    w->events_borrowed = 0;
    w->group_head = 0;
    w->low_resident = 0;
    return NQ_OK;
}

extern "C" nq_status nq_weight_destroy(nq_weight *w)
{
    if (!w) return NQ_ERR_INVALID_ARG;
    if (w->events_borrowed) {   // the head of the group owns the events
        w->low_event = nullptr;
        w->free_event = nullptr;
    }
    if (w->low_event) {
        if (hipEventDestroy((hipEvent_t)w->low_event) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
    }
    if (w->free_event) {
        if (hipEventDestroy((hipEvent_t)w->free_event) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
    }
    w->low_event = nullptr;
    w->free_event = nullptr;
    w->low_event_armed = 0;
    w->free_event_armed = 0;
    w->low_resident = 0;
    return NQ_OK;
}

extern "C" nq_status nq_page_out_low(nq_weight *w, void *stream)
{
    // nothing is moved: the host copy is the master; only the point after which the device
    // slot may be overwritten is marked on `stream`
    if (!w) return NQ_ERR_INVALID_ARG;
    if (w->events_borrowed || w->group_head) return NQ_ERR_INVALID_ARG;   // a group is switched by the batch calls
    if (w->free_event) {
        if (hipEventRecord((hipEvent_t)w->free_event, (hipStream_t)stream) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
        w->free_event_armed = 1;
    }
    w->low_resident = 0;
    w->low_event_armed = 0;
    return NQ_OK;
}

extern "C" nq_status nq_page_in_low(nq_weight *w, void *copy_stream)
{
    if (!w) return NQ_ERR_INVALID_ARG;
    nq_status st = check_cfg(&w->cfg);
    if (st != NQ_OK) return st;
    if (!w->low_event) return NQ_ERR_INVALID_ARG;  // nq_weight_init was not called
    if (w->events_borrowed || w->group_head) return NQ_ERR_INVALID_ARG;   // a group is switched by the batch calls
    const size_t need = nq_packed_bytes(w->N, w->K, low_field_bits(&w->cfg), w->cfg.layout);
    if (w->low_bytes < need) return NQ_ERR_RANGE;
    hipStream_t s = (hipStream_t)copy_stream;
    if (w->free_event_armed && w->free_event) {
        // earlier readers of the slot (full-bit kernels before the page-out) finish first
        if (hipStreamWaitEvent(s, (hipEvent_t)w->free_event, 0) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
        w->free_event_armed = 0;
    }
    if (need > 0) {
        if (!w->d_low || !w->h_low) return NQ_ERR_INVALID_ARG;
        if (!aligned16(w->d_low)) return NQ_ERR_ALIGN;
        if (hipMemcpyAsync(w->d_low, w->h_low, need, hipMemcpyHostToDevice, s) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
    }
    if (hipEventRecord((hipEvent_t)w->low_event, s) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    w->low_event_armed = 1;
    w->low_resident = 1;
    return NQ_OK;
}

// ---- whole-model switching ----------------------------------------------------------------------
extern "C" nq_status nq_weight_init_group(nq_weight *const *ws, int64_t count)
{
    if (!ws || count < 1) return NQ_ERR_INVALID_ARG;
    for (int64_t i = 0; i < count; ++i)
        if (!ws[i]) return NQ_ERR_INVALID_ARG;
    nq_status st = nq_weight_init(ws[0]);
    if (st != NQ_OK) return st;
    ws[0]->group_head = count > 1 ? 1 : 0;
    for (int64_t i = 1; i < count; ++i) {
        nq_weight *w = ws[i];
        if ((st = check_cfg(&w->cfg)) != NQ_OK || (st = check_shape(w->N, w->K)) != NQ_OK) return st;
        const int h = w->cfg.n_bits - w->cfg.l_bits, l = low_field_bits(&w->cfg);
        if (w->high_bytes < nq_packed_bytes(w->N, w->K, h, w->cfg.layout)) return NQ_ERR_RANGE;
        if (w->low_bytes < nq_packed_bytes(w->N, w->K, l, w->cfg.layout)) return NQ_ERR_RANGE;
        if ((w->d_high && !aligned16(w->d_high)) || (w->d_low && !aligned16(w->d_low))) return NQ_ERR_ALIGN;
        w->low_event = ws[0]->low_event;
        w->free_event = ws[0]->free_event;
        w->events_borrowed = 1;
        w->group_head = 0;
        w->low_event_armed = 0;
        w->free_event_armed = 0;
        w->low_resident = 0;
    }
    return NQ_OK;
}

static bool same_group(nq_weight *const *ws, int64_t count)
{
    for (int64_t i = 0; i < count; ++i)
        if (!ws[i] || !ws[i]->low_event || ws[i]->low_event != ws[0]->low_event ||
            ws[i]->free_event != ws[0]->free_event)
            return false;
    return true;
}

extern "C" nq_status nq_page_out_low_batch(nq_weight *const *ws, int64_t count, void *stream)
{
    if (!ws || count < 1) return NQ_ERR_INVALID_ARG;
    if (!same_group(ws, count)) return NQ_ERR_INVALID_ARG;   // not made by nq_weight_init_group
    if (hipEventRecord((hipEvent_t)ws[0]->free_event, (hipStream_t)stream) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    for (int64_t i = 0; i < count; ++i) {
        ws[i]->free_event_armed = 1;
        ws[i]->low_resident = 0;
        ws[i]->low_event_armed = 0;
    }
    return NQ_OK;
}

extern "C" nq_status nq_page_in_low_batch(nq_weight *const *ws, int64_t count, void *copy_stream)
{
    if (!ws || count < 1) return NQ_ERR_INVALID_ARG;
    if (!same_group(ws, count)) return NQ_ERR_INVALID_ARG;
    for (int64_t i = 0; i < count; ++i) {
        nq_status st = check_cfg(&ws[i]->cfg);
        if (st != NQ_OK) return st;
        const size_t need = nq_packed_bytes(ws[i]->N, ws[i]->K, low_field_bits(&ws[i]->cfg), ws[i]->cfg.layout);
        if (ws[i]->low_bytes < need) return NQ_ERR_RANGE;
        if (need > 0 && (!ws[i]->d_low || !ws[i]->h_low)) return NQ_ERR_INVALID_ARG;
        if (need > 0 && !aligned16(ws[i]->d_low)) return NQ_ERR_ALIGN;
    }
    hipStream_t s = (hipStream_t)copy_stream;
    if (ws[0]->free_event_armed) {
        if (hipStreamWaitEvent(s, (hipEvent_t)ws[0]->free_event, 0) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
    }
    // runs of pages that are contiguous on both sides become one copy each
    int64_t i = 0;
    while (i < count) {
        const char *h0 = (const char *)ws[i]->h_low;
        char *d0 = (char *)ws[i]->d_low;
        size_t span = ws[i]->low_bytes;
        int64_t j = i + 1;
        while (j < count && (const char *)ws[j]->h_low == h0 + span && (char *)ws[j]->d_low == d0 + span) {
            span += ws[j]->low_bytes;
            ++j;
        }
        if (j == i + 1) span = nq_packed_bytes(ws[i]->N, ws[i]->K, low_field_bits(&ws[i]->cfg), ws[i]->cfg.layout);
        if (span > 0 && hipMemcpyAsync(d0, h0, span, hipMemcpyHostToDevice, s) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
        i = j;
    }
    if (hipEventRecord((hipEvent_t)ws[0]->low_event, s) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    for (int64_t k = 0; k < count; ++k) {
        ws[k]->free_event_armed = 0;
        ws[k]->low_event_armed = 1;
        ws[k]->low_resident = 1;
    }
    return NQ_OK;
}

// ---- timing events for nq_profile_next_launch ------------------------------------------------
extern "C" nq_status nq_event_create(void **event)
{
    if (!event) return NQ_ERR_INVALID_ARG;
    hipEvent_t ev = nullptr;
    if (hipEventCreate(&ev) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    *event = ev;
    return NQ_OK;
}

extern "C" nq_status nq_event_destroy(void *event)
{
    if (!event) return NQ_ERR_INVALID_ARG;
    if (hipEventDestroy((hipEvent_t)event) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    return NQ_OK;
}

extern "C" nq_status nq_event_elapsed_ms(void *start_event, void *stop_event, float *h_ms)
{
    if (!start_event || !stop_event || !h_ms) return NQ_ERR_INVALID_ARG;
    if (hipEventSynchronize((hipEvent_t)stop_event) != hipSuccess ||
        hipEventElapsedTime(h_ms, (hipEvent_t)start_event, (hipEvent_t)stop_event) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    return NQ_OK;
}
