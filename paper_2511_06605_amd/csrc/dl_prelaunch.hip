// Resident ("prelaunched") kernel and its doorbell: placeholder until the
// protocol lands; every entry reports that no resident kernel is available.
#include "dl_internal.h"

bool dl_resident_running() { return false; }
int dl_resident_submit_plain(const dl_plain_item *, size_t) { return DL_ERR_STATE; }
int dl_resident_submit_fused(const dl_fused_item *, size_t) { return DL_ERR_STATE; }

extern "C" {
int dl_prelaunch_start(void) { return DL_ERR_STATE; }
int dl_prelaunch_stop(void) { return DL_ERR_STATE; }
uint64_t dl_last_ticket(void) { return 0; }
int dl_wait(uint64_t, uint64_t) { return DL_ERR_STATE; }
}
