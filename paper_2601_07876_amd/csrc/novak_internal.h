// Internal declarations shared by the host and device translation units of the NOVAK library.
#ifndef NOVAK_INTERNAL_H_
#define NOVAK_INTERNAL_H_

#include "novak.h"

// chunk sizes are powers of two >= NOVAK_CHUNK_MIN: a chunk splits evenly into the workgroups'
// sub-blocks (1024, 2048 or 4096 elements) and a chunk start keeps a 16-byte aligned tensor aligned
#define NOVAK_CHUNK_MIN 4096
#define NOVAK_CHUNK_MAX (1 << 24)
#define NOVAK_CHUNK_DEFAULT 16384

#endif  // NOVAK_INTERNAL_H_
