// The persistent weight-streaming kernel with residual addition, RMSNorm and the per-token quantiser in front of its
// GEMM (see gemm_decode_resident.hpp, FQ + NORM), with and without SiLU * up behind it: the instantiations for up to
// four tokens and K <= 8192 (the hidden sizes the norm works on), 8 waves.
//
// In a pre-norm decoder layer the linears that read the residual stream (QKV, gate / up) sit behind an addition and a
// norm; at token-generation sizes each of those would be a launch of a few microseconds in front of a GEMM of a few
// microseconds.  Taken into the GEMM's own launch (the fusion policy of Sec. 6.1 taken one operator further; the norm
// itself is LLaMA's) they cost two short passes over a row that already sits in LDS.
#include "gemm_decode_resident.hpp"

namespace w4a8 {

namespace {

template <int XS, int P>
hipError_t launch_norm_p(const DecodeArgs &p, bool swiglu, int grid, int sets, bool prepare_only, hipStream_t stream) {
    if constexpr (epoch_fits(1, XS, P, 8)) {
        if (prepare_only) {
            const hipError_t e = launch_epoch_one<1, XS, P, 8, false, true, 2, true, false, false, true>(p, grid, sets, true, stream);
            return e != hipSuccess ? e : launch_epoch_one<1, XS, P, 8, false, true, 2, true, false, true, true>(p, grid, sets, true, stream);
        }
        return swiglu ? launch_epoch_one<1, XS, P, 8, false, true, 2, true, false, true, true>(p, grid, sets, false, stream)
                      : launch_epoch_one<1, XS, P, 8, false, true, 2, true, false, false, true>(p, grid, sets, false, stream);
    } else {
        return prepare_only ? hipSuccess : hipErrorInvalidConfiguration;
    }
}

}  // namespace

bool decode_norm_supported(int mt, const DecodeShape &s) {
    if (mt != 1 || !s.tiled || !s.fused_quant || s.x_window || s.x_direct || s.aux != 2 || s.k_slices > 1) return false;
    if (s.waves != 8 || s.x_steps < 1 || s.x_steps > 8) return false;
    if (s.prefetch != 1 && s.prefetch != 2) return false;
    if (s.chunk_rows < 4 || s.chunk_rows > 16 || (s.chunk_rows & 3)) return false;
    if (s.rows_per_wg > kResidentMaxRows || (s.rows_per_wg & 3)) return false;
    return epoch_fits(mt, s.x_steps, s.prefetch, s.waves);
}

hipError_t launch_gemm_decode_norm(const DecodeArgs &p, const DecodeShape &s, bool prepare_only, hipStream_t stream) {
    const int grid = prepare_only ? 1 : (p.N + s.rows_per_wg - 1) / s.rows_per_wg;
    const int chunks = prepare_only ? 1 : (s.rows_per_wg + s.chunk_rows - 1) / s.chunk_rows;
    const int sets = chunks > s.prefetch ? 2 : 1;
    hipError_t e = hipSuccess;
#define W4A8_NORM(XS_)                                                                                   \
    if (prepare_only) {                                                                                  \
        if (e == hipSuccess) e = launch_norm_p<XS_, 1>(p, false, grid, sets, true, stream);              \
        if (e == hipSuccess) e = launch_norm_p<XS_, 2>(p, false, grid, sets, true, stream);              \
    } else if (s.x_steps == XS_) {                                                                       \
        return s.prefetch == 2 ? launch_norm_p<XS_, 2>(p, s.swiglu, grid, sets, false, stream)           \
                               : launch_norm_p<XS_, 1>(p, s.swiglu, grid, sets, false, stream);          \
    }
    W4A8_NORM(1) W4A8_NORM(2) W4A8_NORM(3) W4A8_NORM(4) W4A8_NORM(5) W4A8_NORM(6) W4A8_NORM(7) W4A8_NORM(8)
#undef W4A8_NORM
    return prepare_only ? e : hipErrorInvalidConfiguration;
}

}  // namespace w4a8
