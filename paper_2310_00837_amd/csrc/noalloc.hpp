// Set-up of the file-scope scratch array behind helios_dedup_noalloc (noalloc.hip).
#pragma once

namespace helios {

// Looks up the address of the calling thread's current device's copy of the scratch array and keeps
// it for that device; helios_create calls it with the context's device current.  Returns a
// helios_status.
int noalloc_init(int device);

}  // namespace helios
