// Internal declarations shared by the host and device translation units of the NOVAK library.
#ifndef NOVAK_INTERNAL_H_
#define NOVAK_INTERNAL_H_

#include "novak.h"

// chunk sizes are multiples of NOVAK_CHUNK_MIN so that a chunk start keeps a 16-byte aligned
// tensor 16-byte aligned for every element type
#define NOVAK_CHUNK_MIN 1024
#define NOVAK_CHUNK_MAX (1 << 24)
#define NOVAK_CHUNK_DEFAULT 16384

#endif  // NOVAK_INTERNAL_H_
