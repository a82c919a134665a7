// Host-only entry points of libmp8: one Philox4x32-10 block, the loss scaler of Section 3.1
// (arXiv 1905.12334) and status strings.
#include <stdint.h>

#include "../../include/mp8.h"

extern "C" void mp8_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
    uint32_t k[2] = {key[0], key[1]};
    for (int r = 0; r < 10; ++r) {
        const uint64_t a = 0xD2511F53ull * c[0];
        const uint64_t b = 0xCD9E8D57ull * c[2];
        const uint32_t t0 = (uint32_t)(b >> 32) ^ c[1] ^ k[0];
        const uint32_t t2 = (uint32_t)(a >> 32) ^ c[3] ^ k[1];
        c[1] = (uint32_t)b;
        c[3] = (uint32_t)a;
        c[0] = t0;
        c[2] = t2;
        k[0] += 0x9E3779B9u;
        k[1] += 0xBB67AE85u;
    }
    for (int i = 0; i < 4; ++i) out[i] = c[i];
}

extern "C" void mp8_scaler_init(mp8_scaler *s, double scale, double floor, int64_t growth_interval) {
    s->scale = scale < floor ? floor : scale;
    s->floor = floor;
    s->growth_interval = growth_interval < 1 ? 1 : growth_interval;
    s->good_steps = 0;
}

extern "C" int mp8_scaler_update(mp8_scaler *s, uint32_t nonfinite) {
    if (nonfinite != 0) {
        const double halved = s->scale * 0.5;
        s->scale = halved < s->floor ? s->floor : halved;
        s->good_steps = 0;
        return 1;
    }
    if (++s->good_steps >= s->growth_interval) {
        // growth stops at MP8_SCALER_MAX; a scale already beyond it (a floor the caller chose) stays
        if (s->scale < MP8_SCALER_MAX) {
            const double doubled = s->scale * 2.0;
            s->scale = doubled > MP8_SCALER_MAX ? MP8_SCALER_MAX : doubled;
        }
        s->good_steps = 0;
    }
    return 0;
}

extern "C" void mp8_scaler_set_floor(mp8_scaler *s, double floor) {
    s->floor = floor;
    if (s->scale < floor) s->scale = floor;
}

extern "C" const char *mp8_status_string(mp8_status status) {
    switch (status) {
        case MP8_OK: return "ok";
        case MP8_ERR_INVALID_ARG: return "invalid argument";
        case MP8_ERR_UNSUPPORTED: return "unsupported shape or stride";
        case MP8_ERR_ALIGNMENT: return "pointer or leading dimension not 16-byte aligned";
        case MP8_ERR_WORKSPACE: return "workspace missing or too small";
        case MP8_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}
