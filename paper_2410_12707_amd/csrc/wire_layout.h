// Byte arithmetic of the wire message (header | indices, zero-padded to 16 bytes | values), shared
// by the host-only helpers and the kernels' launch code.  Internal to the library.
#ifndef ADATOPK_WIRE_LAYOUT_H
#define ADATOPK_WIRE_LAYOUT_H

#include <stddef.h>
#include <stdint.h>

#include "adatopk.h"

namespace adatopk_internal {

inline bool dtype_ok(adatopk_dtype dt) { return dt == ADATOPK_F32 || dt == ADATOPK_BF16 || dt == ADATOPK_F16; }
inline int elem_size(adatopk_dtype dt) { return dt == ADATOPK_F32 ? 4 : 2; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// first byte of the value section of a message of k pairs
inline size_t wire_val_offset(int64_t k, int index_bytes) {
    return sizeof(adatopk_wire_header) + align_up(static_cast<size_t>(k) * index_bytes, 16);
}

}  // namespace adatopk_internal
#endif
