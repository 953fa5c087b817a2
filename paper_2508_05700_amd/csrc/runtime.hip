// Host-side helpers for callers that have no HIP binding of their own: the
// stream and events of an emb_side_stream, and timing events.  Events made
// here release to device scope only: recording one does not write the caches
// back to system memory, which is all that ordering work between streams of
// one device, or timing it, needs (a default event's system-scope release
// costs microseconds per record and slows the work that follows it).
#include "emb_internal.h"

extern "C" int emb_event_create(void **event_out, int32_t timing)
{
    if (!event_out) return EMB_ERR_INVALID_ARG;
    hipEvent_t e = nullptr;
    const unsigned flags = hipEventReleaseToDevice | (timing ? 0u : (unsigned)hipEventDisableTiming);
    if (hipEventCreateWithFlags(&e, flags) != hipSuccess) return EMB_ERR_HIP;
    *event_out = e;
    return EMB_OK;
}

extern "C" int emb_event_destroy(void *event)
{
    if (!event) return EMB_OK;
    return hipEventDestroy(reinterpret_cast<hipEvent_t>(event)) == hipSuccess ? EMB_OK : EMB_ERR_HIP;
}

extern "C" int emb_event_record(void *event, void *stream)
{
    if (!event) return EMB_ERR_INVALID_ARG;
    return hipEventRecord(reinterpret_cast<hipEvent_t>(event), emb_stream(stream)) == hipSuccess ? EMB_OK : EMB_ERR_HIP;
}

extern "C" int emb_event_elapsed_ms(void *start, void *stop, float *ms_out)
{
    if (!start || !stop || !ms_out) return EMB_ERR_INVALID_ARG;
    return hipEventElapsedTime(ms_out, reinterpret_cast<hipEvent_t>(start), reinterpret_cast<hipEvent_t>(stop)) ==
                   hipSuccess
               ? EMB_OK
               : EMB_ERR_HIP;
}

extern "C" int emb_side_stream_create(emb_side_stream *side)
{
    if (!side) return EMB_ERR_INVALID_ARG;
    side->stream = side->fork_event = side->join_event = nullptr;
    side->defer_join = side->reserved = 0;
    hipStream_t s = nullptr;
    if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) return EMB_ERR_HIP;   // default priority
    side->stream = s;
    if (emb_event_create(&side->fork_event, 0) != EMB_OK || emb_event_create(&side->join_event, 0) != EMB_OK) {
        emb_side_stream_destroy(side);
        return EMB_ERR_HIP;
    }
    return EMB_OK;
}

extern "C" int emb_side_stream_join(const emb_side_stream *side, void *stream)
{
    if (!side || !side->join_event || side->stream == stream) return EMB_ERR_INVALID_ARG;
    return hipStreamWaitEvent(emb_stream(stream), reinterpret_cast<hipEvent_t>(side->join_event), 0) == hipSuccess
               ? EMB_OK
               : EMB_ERR_HIP;
}

extern "C" int emb_side_stream_destroy(emb_side_stream *side)
{
    if (!side) return EMB_ERR_INVALID_ARG;
    int rc = EMB_OK;
    if (side->fork_event && emb_event_destroy(side->fork_event) != EMB_OK) rc = EMB_ERR_HIP;
    if (side->join_event && emb_event_destroy(side->join_event) != EMB_OK) rc = EMB_ERR_HIP;
    if (side->stream && hipStreamDestroy(reinterpret_cast<hipStream_t>(side->stream)) != hipSuccess) rc = EMB_ERR_HIP;
    side->stream = side->fork_event = side->join_event = nullptr;
    return rc;
}
