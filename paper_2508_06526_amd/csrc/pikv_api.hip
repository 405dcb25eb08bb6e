// Host-only parts of the C ABI: descriptor validation, status strings, version.
#include "pikv_common.h"

namespace pikv {

int check_desc(const pikv_desc *d) {
    if (!d) return PIKV_ERR_INVALID;
    if (d->B < 0 || d->Hq < 1 || d->Hkv < 1 || d->E < 1 || d->S < 1 || (d->flags & ~PIKV_DESC_VALUE_BIAS) != 0)
        return PIKV_ERR_INVALID;
    if (d->Hq % d->Hkv != 0) return PIKV_ERR_INVALID;
    if (d->dtype != PIKV_F32 && d->dtype != PIKV_BF16) return PIKV_ERR_INVALID;
    if (d->route_rows_per_seq != 1 && d->route_rows_per_seq != d->Hq) return PIKV_ERR_INVALID;
    if (d->rank < 0 || d->tq < 0 || d->reserved != 0) return PIKV_ERR_INVALID;
    if ((d->flags & PIKV_DESC_VALUE_BIAS) && d->rank == 0) return PIKV_ERR_INVALID;
    if (d->Hq > 256 || d->E > 64) return PIKV_ERR_UNSUPPORTED;
    if (d->D != 16 && d->D != 32 && d->D != 64 && d->D != 128) return PIKV_ERR_UNSUPPORTED;
    if (d->rank != 0 && d->rank != 16 && d->rank != 32 && d->rank != 64) return PIKV_ERR_UNSUPPORTED;
    const int w = desc_width(d);
    const int eb = elem_bytes(d->dtype);
    if (d->stride_s < w || (d->stride_s * eb) % 16 != 0) return PIKV_ERR_INVALID;
    if (d->stride_h < 0 || (d->stride_h * eb) % 16 != 0) return PIKV_ERR_INVALID;
    if (d->Hkv > 1 && d->stride_h < (int64_t)(d->S - 1) * d->stride_s + w) return PIKV_ERR_INVALID;
    return PIKV_OK;
}

}  // namespace pikv

extern "C" const char *pikv_strerror(int status) {
    switch (status) {
        case PIKV_OK: return "ok";
        case PIKV_ERR_INVALID: return "invalid argument";
        case PIKV_ERR_UNSUPPORTED: return "shape not supported by the gfx950 kernels";
        case PIKV_ERR_WORKSPACE: return "workspace too small";
        case PIKV_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

extern "C" int pikv_version(void) { return 301; }
