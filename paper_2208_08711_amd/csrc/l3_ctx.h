/*
 * The context object behind the opaque l3_ctx of include/l3.h, shared by the
 * translation units that enqueue GPU work.  Not part of the public ABI.
 */
#ifndef L3_CTX_H
#define L3_CTX_H

#include <hip/hip_runtime.h>

#include "l3_internal.h"

constexpr int kSlots = 4;   /* descriptor staging slots: calls in flight before the host waits */

struct L3EncodeState;                          /* workspace of l3_encode_batch, owned by its file */
void l3_encode_state_free(L3EncodeState* s);   /* NULL allowed */

struct L3AblationState;                        /* workspace of l3_ablation_decode_batch */
void l3_ablation_state_free(L3AblationState* s);   /* NULL allowed */

struct l3_ctx {
    int device = 0;
    L3ImageDesc* scratch = nullptr;       /* host: descriptors of the call being planned */
    size_t scratch_cap = 0;
    size_t cap = 0;                       /* descriptors per slot */
    L3ImageDesc* h_stage[kSlots] = {};    /* pinned host */
    L3ImageDesc* d_descs[kSlots] = {};    /* device */
    bool flat_order = true;               /* flat order of work units allowed (L3_FLAT_ORDER=0 at creation: off) */
    /* Fused path: tables of the 256 normalised values per channel, one slot per (constants,
     * stream) pair in use; table_used[s] is recorded behind every call that reads slot s, so
     * that a call on another stream that takes the slot over can wait for it on the device. */
    uint16_t* d_table[kSlots] = {};       /* device: 768 entries each */
    uint16_t* d_table_capture = nullptr;  /* device: the table of calls made under stream capture */
    float table_key[kSlots][7] = {};      /* mean, stdv, dtype the slot's table was built with */
    bool table_valid[kSlots] = {};
    hipStream_t table_stream[kSlots] = {};
    hipEvent_t table_used[kSlots] = {};
    bool table_used_valid[kSlots] = {};
    int table_cur = 0;                    /* the slot the last fused call used */
    uint16_t* static_table = nullptr;     /* device: this GPU's copy of the library's static table */
    hipEvent_t done[kSlots] = {};         /* the slot's kernels have finished */
    bool pending[kSlots] = {};
    int next = 0;
    L3EncodeState* enc = nullptr;
    L3AblationState* abl = nullptr;
};

/* Makes the context's device current for the lifetime of the guard. */
struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int device) {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = prev == device || hipSetDevice(device) == hipSuccess;
    }
    ~DeviceGuard() {
        int now = -1;
        if (prev >= 0 && hipGetDevice(&now) == hipSuccess && now != prev) (void)hipSetDevice(prev);
    }
};

#endif
