// Host-only part of libtetri that needs no HIP: chunk packer, scheduler, per-chunk metadata.
#pragma once
#include "tetri.h"

// Message of the calling thread's last failed call that had no handle to keep it in.
void tetri_set_thread_error(const char *msg);
const char *tetri_thread_error();
