// bf16 MFMA path (placeholder until the kernels land): reports nothing as supported.
#include "flurka_internal.h"

namespace flurka {

bool fast_supported(const Problem&, int) { return false; }

bool fast_pointers_ok(const void* a, const void* b, const void* c, const void* d, const void* e,
                      const void* f, const void* g) {
    const void* ps[7] = {a, b, c, d, e, f, g};
    for (const void* p : ps)
        if (p && ((uintptr_t)p % 16) != 0) return false;
    return true;
}

size_t fast_ws_bytes(const Problem&, int) { return 0; }

flurka_status fast_forward(const Problem&, const FwdArgs&, hipStream_t) { return FLURKA_ERR_UNSUPPORTED; }
flurka_status fast_backward(const Problem&, const BwdArgs&, hipStream_t) { return FLURKA_ERR_UNSUPPORTED; }

}  // namespace flurka
