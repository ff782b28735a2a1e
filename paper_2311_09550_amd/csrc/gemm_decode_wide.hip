// The persistent weight-streaming kernel for up to 64 tokens: instantiations in which every wave stages its own k
// steps of the activations through a window of LDS (see gemm_decode_resident.hpp), over the tiled weight array.
//
// Between token generation proper and the large-M tiling lies the range where a GEMM is still bound by the one pass
// over the weights (Sec. 4.1 puts the self-decoding stage on the memory-bound side), but the activations no longer fit
// beside them: an LDS-staged tiling re-reads them per tile and spends most of a compute unit's outstanding loads on
// them.  Here they sit in registers, 16 MT rows x XS k steps per wave, and every outstanding load is a weight load.
#include "gemm_decode_resident.hpp"

namespace w4a8 {

namespace {

template <int MT, int XS, int P, int WAVES>
hipError_t launch_wide_p(const DecodeArgs &p, bool acc_out, int grid, int sets, bool prepare_only, hipStream_t stream) {
    if constexpr (epoch_fits(MT, XS, P, WAVES)) {
        if (prepare_only) {
            const hipError_t e = launch_epoch_one<MT, XS, P, WAVES, false, true, 2, false, true>(p, grid, sets, true, stream);
            return e != hipSuccess ? e : launch_epoch_one<MT, XS, P, WAVES, true, true, 2, false, true>(p, grid, sets, true, stream);
        }
        return acc_out ? launch_epoch_one<MT, XS, P, WAVES, true, true, 2, false, true>(p, grid, sets, false, stream)
                       : launch_epoch_one<MT, XS, P, WAVES, false, true, 2, false, true>(p, grid, sets, false, stream);
    } else {
        return prepare_only ? hipSuccess : hipErrorInvalidConfiguration;
    }
}

}  // namespace

bool decode_wide_supported(int mt, const DecodeShape &s) {
    if (!s.tiled || s.fused_quant || s.x_direct || s.aux != 2) return false;
    if (s.prefetch != 1 && s.prefetch != 2) return false;
    if (s.chunk_rows < 4 || s.chunk_rows > 16 || (s.chunk_rows & 3)) return false;
    if (s.rows_per_wg > kResidentMaxRows) return false;
    return wide_shape_exists(mt, s.x_steps, s.waves) && epoch_fits(mt, s.x_steps, s.prefetch, s.waves);
}

hipError_t launch_gemm_decode_wide(const DecodeArgs &p, bool acc_out, const DecodeShape &s, int mt, bool prepare_only,
                                   hipStream_t stream) {
    const int grid = prepare_only ? 1 : (p.N + s.rows_per_wg - 1) / s.rows_per_wg;
    const int chunks = prepare_only ? 1 : (s.rows_per_wg + s.chunk_rows - 1) / s.chunk_rows;
    const int sets = chunks > s.prefetch ? 2 : 1;
    hipError_t e = hipSuccess;
#define W4A8_WIDE(MT_, XS_, WV_)                                                                              \
    static_assert(wide_shape_exists(MT_, XS_, WV_), "the table and the check must agree");                    \
    if (prepare_only) {                                                                                       \
        if (e == hipSuccess) e = launch_wide_p<MT_, XS_, 1, WV_>(p, acc_out, grid, sets, true, stream);       \
        if (e == hipSuccess) e = launch_wide_p<MT_, XS_, 2, WV_>(p, acc_out, grid, sets, true, stream);       \
    } else if (mt == MT_ && s.x_steps == XS_ && s.waves == WV_) {                                             \
        return s.prefetch == 2 ? launch_wide_p<MT_, XS_, 2, WV_>(p, acc_out, grid, sets, false, stream)       \
                               : launch_wide_p<MT_, XS_, 1, WV_>(p, acc_out, grid, sets, false, stream);      \
    }
    W4A8_WIDE(1, 1, 8) W4A8_WIDE(1, 2, 8) W4A8_WIDE(1, 3, 8) W4A8_WIDE(1, 4, 8) W4A8_WIDE(1, 5, 8) W4A8_WIDE(1, 6, 8)
    W4A8_WIDE(1, 7, 8) W4A8_WIDE(1, 8, 8) W4A8_WIDE(1, 11, 8) W4A8_WIDE(1, 14, 8)
    W4A8_WIDE(1, 5, 16) W4A8_WIDE(1, 6, 16) W4A8_WIDE(1, 7, 16) W4A8_WIDE(1, 8, 16)
    W4A8_WIDE(2, 1, 16) W4A8_WIDE(2, 2, 16) W4A8_WIDE(2, 3, 16) W4A8_WIDE(2, 4, 16)
    W4A8_WIDE(2, 1, 8) W4A8_WIDE(2, 2, 8) W4A8_WIDE(2, 3, 8) W4A8_WIDE(2, 4, 8) W4A8_WIDE(2, 5, 8) W4A8_WIDE(2, 6, 8)
    W4A8_WIDE(2, 7, 8)
    W4A8_WIDE(3, 1, 8) W4A8_WIDE(3, 2, 8) W4A8_WIDE(3, 3, 8) W4A8_WIDE(3, 4, 8) W4A8_WIDE(3, 5, 8)
    W4A8_WIDE(4, 1, 8) W4A8_WIDE(4, 2, 8) W4A8_WIDE(4, 3, 8) W4A8_WIDE(4, 4, 8) W4A8_WIDE(4, 5, 8)
#undef W4A8_WIDE
    return prepare_only ? e : hipErrorInvalidConfiguration;
}

}  // namespace w4a8
