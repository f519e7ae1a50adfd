// placeholder until the fused kernel lands
#include "fftconv_internal.h"
namespace fftconv {
bool fused3_supported(int64_t, int64_t, int) { return false; }
int fused3_init(fftconv_plan *) { return FFTCONV_EUNSUPPORTED; }
void fused3_destroy(fftconv_plan *) {}
size_t fused3_kf_bytes(const fftconv_plan *) { return 0; }
int fused3_pack_kf(const fftconv_plan *, const double2 *, int64_t, int64_t, const uint8_t *, int64_t, void *, hipStream_t) { return FFTCONV_EUNSUPPORTED; }
int fused3_forward(const fftconv_plan *, const void *, const void *, void *, int64_t, hipStream_t) { return FFTCONV_EUNSUPPORTED; }
}
