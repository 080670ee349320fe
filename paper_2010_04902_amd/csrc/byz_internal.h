// Shared between the translation units of libbyzshield (not part of the C-ABI).
#ifndef BYZ_INTERNAL_H
#define BYZ_INTERNAL_H

// Records the hipError_t that byz_last_hip_error() reports for the calling thread.
void byz_internal_set_hip_error(int code);

#endif
