// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/dmalatte.h"
#include "dl_work.h"

// Library state (one device, one host thread).
struct dl_state {
    bool inited = false;
    int device = -1;
    int num_cu = 0;
    int mode = DL_MODE_ONESHOT;
    int validate = 0;
    int last_hip = 0;
    dl_config cfg{};
};
extern dl_state g_dl;

#define DL_HIP(call)                                  \
    do {                                              \
        hipError_t e_ = (call);                       \
        if (e_ != hipSuccess) {                       \
            g_dl.last_hip = (int)e_;                  \
            (void)hipGetLastError();                  \
            return DL_ERR_HIP;                        \
        }                                             \
    } while (0)

// Launch geometry chosen on the host for one request.
struct dl_launch_shape {
    uint32_t tile_bytes;
    uint32_t block_threads;
    uint32_t max_blocks;  // 0 = one workgroup per tile
    bool nontemporal;
};

// dl_exec.hip: one-shot execution of a lowered list on a stream.
int dl_exec_plain(const dl_plain_item *items, size_t n, hipStream_t stream);
int dl_exec_fused(const dl_fused_item *items, size_t n, hipStream_t stream);
int dl_exec_init();
int dl_exec_shutdown();
dl_launch_shape dl_choose_shape(uint64_t src_bytes, uint64_t max_item_bytes, uint32_t max_k);

// dl_prelaunch.hip: the resident kernel and its doorbell.
int dl_resident_submit_plain(const dl_plain_item *items, size_t n);
int dl_resident_submit_fused(const dl_fused_item *items, size_t n);
bool dl_resident_running();
