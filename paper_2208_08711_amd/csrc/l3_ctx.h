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
    /* Fused path: the table of normalised values of the last call's constants (host memory;
     * it travels in the kernel arguments) */
    uint16_t table_bits[768] = {};
    float table_key[7] = {};              /* mean, stdv, dtype it was worked out for */
    bool table_valid = false;
    uint32_t resident_workgroups = 2048;  /* workgroups of a launch's last round (8 per CU) */
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
