// Specialised codec kernels (placeholder: nothing is specialised yet, every call takes the generic kernels).
#include "pbz_internal.h"

namespace pbz {

int try_compress_fast(const pbz_codec*, const Geom&, const void*, int, void*, void*, hipStream_t, bool, const char**) {
  return 0;
}

int try_decompress_fast(const pbz_codec*, const Geom&, const void*, const void*, void*, int, hipStream_t, bool,
                        const char**) {
  return 0;
}

}  // namespace pbz
