// Host-side marker/table parser of libprep (T.81 Annex B).
#pragma once
#include <stdint.h>

#include "../../include/prep.h"

namespace prep {

struct ParsedImage {
    prep_image_info info;
    uint32_t dht_off[4];   // BITS[16] of DC luma, AC luma, DC chroma, AC chroma (from file start)
    uint32_t dht_nval[4];
    uint32_t dqt_off[3];   // 64 zig-zag ordered quantiser bytes per component
};

// Parse one file.  Returns and stores in out->info.status PREP_OK,
// PREP_E_UNSUPPORTED or PREP_E_CORRUPT; never reads outside [d, d+len).
int parse_image(const uint8_t *d, uint64_t len, ParsedImage *out);

}  // namespace prep
