// Dynamic buffer manager (Section 3.2): host logic only.  Buffers are carved, one after the other, out
// of a caller-owned arena of device memory that the manager never dereferences; a request is served
// from the list of buffers created so far when the section's rules allow it:
//   within a module   an idle buffer is reused only when its size equals the request;
//   across modules    the first idle buffer that is large enough is reused.
// A buffer belongs to the module that used it last.  Nothing is ever handed back to the arena: the
// list only grows until the working set of a forward pass has been seen once, after which every
// request is a reuse (no allocation on the hot path, Section 3.1).
#include "../../include/eet.h"

#include <cstdarg>
#include <cstdio>
#include <new>
#include <vector>

int eet_set_error(int code, const char* fmt, ...);   // eet_api.hip

namespace {
struct Buffer {
    size_t offset, size;
    int32_t module;
    bool idle;
};
}  // namespace

struct eet_bufmgr {
    char* arena;
    size_t arena_bytes, footprint;
    std::vector<Buffer> list;          // creation order
    int64_t requests, same_size, larger, created;
};

static constexpr size_t kAlign = 256;

extern "C" {

int eet_bufmgr_create(void* arena, size_t arena_bytes, eet_bufmgr_t** out) {
    if (!out) return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_create: out is null");
    *out = nullptr;
    if (!arena || arena_bytes == 0) return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_create: empty arena");
    if (reinterpret_cast<uintptr_t>(arena) % kAlign != 0)
        return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_create: the arena must be 256-byte aligned");
    eet_bufmgr* m = new (std::nothrow) eet_bufmgr{static_cast<char*>(arena), arena_bytes, 0, {}, 0, 0, 0, 0};
    if (!m) return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_create: out of host memory");
    *out = m;
    return EET_OK;
}

int eet_bufmgr_request(eet_bufmgr_t* m, size_t bytes, int32_t module, void** out) {
    if (!m || !out) return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_request: null argument");
    *out = nullptr;
    if (bytes == 0) return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_request: zero bytes requested");
    if (bytes > m->arena_bytes) return eet_set_error(EET_ERR_CAPACITY, "eet_bufmgr_request: %zu bytes exceed the arena", bytes);
    const size_t size = (bytes + kAlign - 1) / kAlign * kAlign;
    for (Buffer& b : m->list) {
        if (!b.idle) continue;
        const bool same_module = b.module == module;
        if (same_module ? b.size != size : b.size < size) continue;
        b.idle = false;
        b.module = module;
        ++m->requests;
        ++(b.size == size ? m->same_size : m->larger);
        *out = m->arena + b.offset;
        return EET_OK;
    }
    if (size > m->arena_bytes - m->footprint)
        return eet_set_error(EET_ERR_CAPACITY, "eet_bufmgr_request: %zu bytes do not fit: %zu of %zu in use", size, m->footprint,
                             m->arena_bytes);
    try {
        m->list.push_back(Buffer{m->footprint, size, module, false});
    } catch (const std::bad_alloc&) {
        return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_request: out of host memory");
    }
    *out = m->arena + m->footprint;
    m->footprint += size;
    ++m->requests;
    ++m->created;
    return EET_OK;
}

int eet_bufmgr_release(eet_bufmgr_t* m, void* buffer) {
    if (!m || !buffer) return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_release: null argument");
    for (Buffer& b : m->list) {
        if (m->arena + b.offset != buffer) continue;
        if (b.idle) return eet_set_error(EET_ERR_STATE, "eet_bufmgr_release: the buffer is already idle");
        b.idle = true;
        return EET_OK;
    }
    return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_release: not a buffer of this manager");
}

int eet_bufmgr_query(const eet_bufmgr_t* m, eet_bufmgr_stats* out) {
    if (!m || !out) return eet_set_error(EET_ERR_INVALID_ARG, "eet_bufmgr_query: null argument");
    out->arena_bytes = m->arena_bytes;
    out->footprint_bytes = m->footprint;
    out->buffers = (int64_t)m->list.size();
    out->idle = 0;
    for (const Buffer& b : m->list) out->idle += b.idle ? 1 : 0;
    out->requests = m->requests;
    out->reused_same_size = m->same_size;
    out->reused_larger = m->larger;
    out->created = m->created;
    return EET_OK;
}

int eet_bufmgr_destroy(eet_bufmgr_t* m) {
    delete m;
    return EET_OK;
}

}  // extern "C"
