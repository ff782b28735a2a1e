// The persistent weight-streaming kernel with SiLU * up in its epilogue (see gemm_decode_resident.hpp, SWIGLU): the
// instantiations over the interleaved gate / up weights, with the fused per-token quantiser (up to four tokens, fp16
// activations in) and with per-wave staging (up to 64 tokens, quantised activations in).
//
// At token-generation sizes a layer is a handful of launches of a few microseconds each, and the row-wise SiLU * up
// kernel between the gate / up projection and the down projection is one of them; folded into the projection's
// epilogue (the fusion policy of Sec. 6.1) it costs two exponentials per lane and the launch disappears, as do the
// write and the read of the M x 2 I intermediate.
#include "gemm_decode_resident.hpp"

namespace w4a8 {

namespace {

template <int XS, int P, int WAVES>
hipError_t launch_fused_p(const DecodeArgs &p, int grid, int sets, bool prepare_only, hipStream_t stream) {
    if constexpr (epoch_fits(1, XS, P, WAVES))
        return launch_epoch_one<1, XS, P, WAVES, false, true, 2, true, false, true>(p, grid, sets, prepare_only, stream);
    else
        return prepare_only ? hipSuccess : hipErrorInvalidConfiguration;
}

template <int MT, int XS, int P, int WAVES>
hipError_t launch_window_p(const DecodeArgs &p, int grid, int sets, bool prepare_only, hipStream_t stream) {
    if constexpr (epoch_fits(MT, XS, P, WAVES))
        return launch_epoch_one<MT, XS, P, WAVES, false, true, 2, false, true, true>(p, grid, sets, prepare_only, stream);
    else
        return prepare_only ? hipSuccess : hipErrorInvalidConfiguration;
}

}  // namespace

bool decode_swiglu_supported(int mt, const DecodeShape &s) {
    if (!s.tiled || s.x_direct || s.aux != 2 || s.k_slices > 1) return false;
    if (s.prefetch != 1 && s.prefetch != 2) return false;
    if (s.chunk_rows < 4 || s.chunk_rows > 16 || (s.chunk_rows & 3)) return false;
    if (s.rows_per_wg > kResidentMaxRows || (s.rows_per_wg & 3)) return false;
    if (s.fused_quant)
        return !s.x_window && mt == 1 && fused_shape_exists(s.x_steps, s.waves) && epoch_fits(mt, s.x_steps, s.prefetch, s.waves);
    return s.x_window && mt <= 4 && decode_wide_supported(mt, s);
}

hipError_t launch_gemm_decode_swiglu(const DecodeArgs &p, const DecodeShape &s, int mt, bool prepare_only, hipStream_t stream) {
    const int grid = prepare_only ? 1 : (p.N + s.rows_per_wg - 1) / s.rows_per_wg;
    const int chunks = prepare_only ? 1 : (s.rows_per_wg + s.chunk_rows - 1) / s.chunk_rows;
    const int sets = chunks > s.prefetch ? 2 : 1;
    hipError_t e = hipSuccess;
#define W4A8_FUSED(XS_, WV_)                                                                          \
    static_assert(fused_shape_exists(XS_, WV_), "the table and the check must agree");                \
    if (prepare_only) {                                                                               \
        if (e == hipSuccess) e = launch_fused_p<XS_, 1, WV_>(p, grid, sets, true, stream);            \
        if (e == hipSuccess) e = launch_fused_p<XS_, 2, WV_>(p, grid, sets, true, stream);            \
    } else if (s.fused_quant && mt == 1 && s.x_steps == XS_ && s.waves == WV_) {                      \
        return s.prefetch == 2 ? launch_fused_p<XS_, 2, WV_>(p, grid, sets, false, stream)            \
                               : launch_fused_p<XS_, 1, WV_>(p, grid, sets, false, stream);           \
    }
    W4A8_FUSED(1, 8) W4A8_FUSED(2, 8) W4A8_FUSED(3, 8) W4A8_FUSED(4, 8) W4A8_FUSED(5, 8) W4A8_FUSED(6, 8) W4A8_FUSED(7, 8)
    W4A8_FUSED(8, 8) W4A8_FUSED(11, 8) W4A8_FUSED(14, 8)
    W4A8_FUSED(1, 16) W4A8_FUSED(2, 16) W4A8_FUSED(3, 16) W4A8_FUSED(4, 16) W4A8_FUSED(5, 16) W4A8_FUSED(6, 16)
    W4A8_FUSED(7, 16) W4A8_FUSED(8, 16)
#undef W4A8_FUSED
#define W4A8_WINDOW(MT_, XS_, WV_)                                                                    \
    static_assert(wide_shape_exists(MT_, XS_, WV_), "the table and the check must agree");            \
    if (prepare_only) {                                                                               \
        if (e == hipSuccess) e = launch_window_p<MT_, XS_, 1, WV_>(p, grid, sets, true, stream);      \
        if (e == hipSuccess) e = launch_window_p<MT_, XS_, 2, WV_>(p, grid, sets, true, stream);      \
    } else if (s.x_window && mt == MT_ && s.x_steps == XS_ && s.waves == WV_) {                       \
        return s.prefetch == 2 ? launch_window_p<MT_, XS_, 2, WV_>(p, grid, sets, false, stream)      \
                               : launch_window_p<MT_, XS_, 1, WV_>(p, grid, sets, false, stream);     \
    }
    W4A8_WINDOW(1, 1, 8) W4A8_WINDOW(1, 2, 8) W4A8_WINDOW(1, 3, 8) W4A8_WINDOW(1, 4, 8) W4A8_WINDOW(1, 5, 8)
    W4A8_WINDOW(1, 6, 8) W4A8_WINDOW(1, 7, 8) W4A8_WINDOW(1, 8, 8) W4A8_WINDOW(1, 11, 8) W4A8_WINDOW(1, 14, 8)
    W4A8_WINDOW(1, 5, 16) W4A8_WINDOW(1, 6, 16) W4A8_WINDOW(1, 7, 16) W4A8_WINDOW(1, 8, 16)
    W4A8_WINDOW(2, 1, 16) W4A8_WINDOW(2, 2, 16) W4A8_WINDOW(2, 3, 16) W4A8_WINDOW(2, 4, 16)
    W4A8_WINDOW(2, 1, 8) W4A8_WINDOW(2, 2, 8) W4A8_WINDOW(2, 3, 8) W4A8_WINDOW(2, 4, 8) W4A8_WINDOW(2, 5, 8)
    W4A8_WINDOW(2, 6, 8) W4A8_WINDOW(2, 7, 8)
    W4A8_WINDOW(3, 1, 8) W4A8_WINDOW(3, 2, 8) W4A8_WINDOW(3, 3, 8) W4A8_WINDOW(3, 4, 8) W4A8_WINDOW(3, 5, 8)
    W4A8_WINDOW(4, 1, 8) W4A8_WINDOW(4, 2, 8) W4A8_WINDOW(4, 3, 8) W4A8_WINDOW(4, 4, 8) W4A8_WINDOW(4, 5, 8)
#undef W4A8_WINDOW
    return prepare_only ? e : hipErrorInvalidConfiguration;
}

}  // namespace w4a8
