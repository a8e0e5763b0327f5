// Host-side helpers shared by the launch-sequence builders (internal).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <vector>

#include "../../include/tsr.h"

namespace tsr {

int& last_hip_error();

inline int hip_fail(hipError_t e) {
    last_hip_error() = (int)e;
    return TSR_HIP_ERROR;
}
#define TSR_HIP(call)                                  \
    do {                                               \
        hipError_t e__ = (call);                       \
        if (e__ != hipSuccess) return hip_fail(e__);   \
    } while (0)
#define TSR_TRY(call)                    \
    do {                                 \
        int s__ = (call);                \
        if (s__ != TSR_OK) return s__;   \
    } while (0)

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Bump allocator over the caller's workspace.  With base == nullptr it only measures.
struct Arena {
    char* base;
    size_t off = 0;
    explicit Arena(void* b) : base((char*)b) {}
    template <typename T> T* take(size_t count) {
        off = align_up(off);
        T* p = base ? (T*)(base + off) : (T*)nullptr;
        off += count * sizeof(T);
        return p;
    }
    size_t used() const { return align_up(off); }
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Optional per-stage timing: HIP events recorded on the work stream around every stage.
struct Prof {
    struct Span { int kind; hipEvent_t a, b; };
    std::vector<Span> spans;
    bool on = false;
    void clear() {
        for (Span& s : spans) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
        spans.clear();
    }
};

struct Ctx {                  // where to enqueue, and whether to time it
    hipStream_t s;
    Prof* prof;
};

struct Timed {                // RAII bracket of one stage
    Ctx& c; int idx = -1;
    Timed(Ctx& ctx, int kind) : c(ctx) {
        if (c.prof && c.prof->on) {
            Prof::Span sp{kind, nullptr, nullptr};
            if (hipEventCreate(&sp.a) == hipSuccess && hipEventCreate(&sp.b) == hipSuccess) {
                (void)hipEventRecord(sp.a, c.s);
                c.prof->spans.push_back(sp);
                idx = (int)c.prof->spans.size() - 1;
            }
        }
    }
    ~Timed() { if (idx >= 0) (void)hipEventRecord(c.prof->spans[idx].b, c.s); }
};

// Device tables, carved from the arena after every data buffer and mirrored in `host`
// (host[0] corresponds to arena offset `first`) so that one copy uploads them all.
struct Uploader {
    std::vector<char> host;
    size_t first = (size_t)-1;
    template <typename T> const T* put(const std::vector<T>& v, Arena& ar) {
        T* d = ar.take<T>(v.size());
        if (ar.base) {
            const size_t o = (size_t)((char*)d - ar.base);
            if (first == (size_t)-1) first = o;
            const size_t rel = o - first;
            if (host.size() < rel + v.size() * sizeof(T)) host.resize(rel + v.size() * sizeof(T));
            if (!v.empty()) memcpy(host.data() + rel, v.data(), v.size() * sizeof(T));
        }
        return d;
    }
};


struct BlockView {          // what the step needs to know about one block
    const void* G; int g_dtype; int m, n, r; long long ldg, g_stride;
    float* W; long long ldw; float* U; float* V; float* M; float* Vm; float* C; float* D;
};


}  // namespace tsr
