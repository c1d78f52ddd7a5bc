// Catch-up ("prefix") pass over a chunk of tokens.  Bring-up version: the definition itself,
// one single-token step per row.
#include "st_device.h"
#include "st_internal.h"

namespace st {

void launch_prefill_layers(const Model &m, int32_t pos0, int32_t n) {
    for (int32_t i = 0; i < n; ++i) {
        launch_set_state(m, kPos, pos0 + i);
        launch_set_token_from(m, m.ws.tokens, i);
        launch_decode_layers(m, m.ws.x + (size_t)i * m.c.hidden);
    }
    launch_set_state(m, kPos, pos0);
}

}  // namespace st
