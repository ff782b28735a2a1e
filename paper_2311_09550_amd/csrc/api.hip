// C ABI of the W4A8 library: argument validation, tiling choice, launches.
// Nothing here touches the data; every step of the path runs in the kernels.
#include "../../include/w4a8.h"
#include "../../include/w4a8_tuning.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

#include "kernels.hpp"

namespace {

using namespace w4a8;

constexpr int kDecodeMaxM = 64;

// What HIP said when an entry point last returned W4A8_ERR_LAUNCH on this thread (hipSuccess if it never did).
thread_local hipError_t last_hip_error = hipSuccess;

inline int launched(hipError_t e) {
    if (e == hipSuccess) return W4A8_OK;
    last_hip_error = e;
    (void)hipGetLastError();  // a rejected launch leaves its error in the runtime's per-thread slot: take it out
    return W4A8_ERR_LAUNCH;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline int check_gemm_shape(int M, int N, int K) {
    if (M < 1 || N < 1 || K < 32 || (K % 32) != 0 || K > W4A8_MAX_K) return W4A8_ERR_SHAPE;
    return W4A8_OK;
}

// Compute units of the current device (256 on MI355X); queried once per device.
int compute_units() {
    static std::atomic<int> cus[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Scratch memory of the entry point that allocates nothing (w4a8_gemm_tiled_splitk_static): the slabs of raw sums
// that the K slices of one GEMM exchange.  One array per GPU, held from the moment the library is loaded until the
// process ends.  `scratch` is only the host-side name of the symbol; the device address is looked up once per device
// and every use below goes through that address.
constexpr size_t kStaticScratchBytes = W4A8_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (NULL and an error code if the lookup fails).
int static_scratch(void **ptr) {
    static void *addr[kMaxDevices];
    static std::atomic<bool> known[kMaxDevices];
    static std::mutex lookup_lock;
    int dev = 0;
    *ptr = nullptr;
    if (int e = launched(hipGetDevice(&dev))) return e;
    if (dev < 0 || dev >= kMaxDevices) return launched(hipErrorInvalidDevice);
    if (!known[dev].load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> hold(lookup_lock);
        if (!known[dev].load(std::memory_order_relaxed)) {
            void *p = nullptr;
            if (int e = launched(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)))) return e;
            if (p == nullptr) return launched(hipErrorInvalidSymbol);
            addr[dev] = p;
            known[dev].store(true, std::memory_order_release);
        }
    }
    *ptr = addr[dev];
    return W4A8_OK;
}

struct Plan {
    int tiling;
    DecodeShape decode;
    int prefill_tile;
};

bool resident_shape(int M, int N, int K, int waves, int grid, int prefetch, bool whole16, int aux, bool tiled, DecodeShape *out,
                    int k_slices = 1, bool x_window = false);

// 17 to 64 tokens over tiled weights: shape of the persistent kernel with per-wave staging, cut into the fewest K
// slices for which an instantiation exists (slices_forced > 0: exactly that many).  False when there is none.
bool wide_plan(int M, int N, int K, int slices_forced, int max_slices, DecodeShape *out) {
    if (M <= 16 || M > kResidentMaxM) return false;
    const int first = slices_forced > 0 ? slices_forced : 1, last = slices_forced > 0 ? slices_forced : max_slices;
    for (int s = first; s <= last; ++s) {
        DecodeShape t{};
        if (resident_shape(M, N, K, 0, 0, 0, false, -1, true, &t, s, true)) {
            *out = t;
            return true;
        }
    }
    return false;
}

// Shape of the persistent weight-streaming kernel for (M, N, K).  Returns false when a wave's share of the
// activations would not fit in registers (then the general streaming kernel takes over).
//   waves    : 8 or 16, 0 = library's choice (8 wherever a wave's k steps fit its registers, see below);
//   grid     : workgroups wanted, 0 = library's choice.  A workgroup's range is N / grid rounded up to whole cache
//              lines of the weight array (8 channels in the tiled array, 4 in the row-major one).  The library's own
//              choice is one workgroup per compute unit with the range rounded up to whole 16-channel chunks
//              (measured on LLaMA-7B/13B/70B shapes, cold weights: within 4 % of the best grid everywhere; ranges of
//              20 or 24 channels, i.e. chunks of 12, lose up to 13 % to ranges of 32 on fewer compute units);
//   prefetch : chunks of weight loads a wave keeps in flight, 0 = library's choice: one, since a compute unit takes
//              only some 40 to 50 outstanding wave-wide loads and one chunk per wave already is that many; two where a
//              range is exactly two chunks and M <= 8 (everything is then requested at once: 4 to 5 % on 13B's O;
//              level at 16 tokens, slower on every other shape tried);
//   whole16  : chunks of 16 channels even where the range does not divide evenly;
//   aux      : cache policy of the weight loads, -1 = library's choice (non-temporal: 5 to 10 % faster);
//   k_slices : workgroups along K (raw sums only when more than one);
//   x_window : every wave stages its own k steps (tiled weights, 17 to 64 tokens).  Then waves = 0 means 16 waves for
//              two column tiles when their k steps fit, else 8.
bool resident_shape(int M, int N, int K, int waves, int grid, int prefetch, bool whole16, int aux, bool tiled, DecodeShape *out,
                    int k_slices, bool x_window) {
    const int mt = (M + 15) / 16;
    DecodeShape s{};
    s.resident = true;
    s.tiled = tiled;
    s.fused_quant = out->fused_quant;  // set by the caller that wants the kernel to quantise its own activations
    s.swiglu = out->swiglu;            // ... or to apply SiLU * up to interleaved gate / up channels
    s.norm = out->norm;                // ... or to add the residual and normalise in front of its quantiser
    s.aux = aux < 0 ? 2 : aux;
    s.x_window = x_window;
    s.k_slices = k_slices < 1 ? 1 : k_slices;
    const int ks_total = ((K + 127) / 128 + s.k_slices - 1) / s.k_slices;  // k steps of a slice
    // 8 waves wherever their k steps fit the registers (measured 4 to 13 % faster than 16): up to 14 steps per wave
    // for one column tile (K <= 14336), 7 for two with per-wave staging, 5 for three and four
    if (waves == 0) {
        if (mt == 1)
            waves = ks_total <= 112 ? 8 : 16;
        else if (x_window)
            waves = (mt == 2 && ks_total > 56) ? 16 : 8;
        else
            waves = 16;
    }
    s.waves = waves;
    s.x_steps = (ks_total + waves - 1) / waves;
    // beyond 8 steps per wave only 11 and 14 are instantiated; a wave's surplus steps load nothing and multiply zeros
    if (mt == 1 && waves == 8 && s.x_steps > 8) s.x_steps = s.x_steps <= 11 ? 11 : 14;
    // In the tiled array a 128-byte line holds 16 bytes of each of 8 consecutive channels: ranges that start on
    // multiples of 8 channels never share a line with a neighbour (which would fetch it a second time).
    const int unit = tiled ? 8 : 4;
    int rows;
    if (grid <= 0) {
        const long long per_wg = ((long long)N * s.k_slices + compute_units() - 1) / compute_units();
        rows = per_wg > kResidentMaxRows ? kResidentMaxRows : (int)((per_wg + 15) / 16 * 16);
        if (rows > kResidentMaxRows) rows = kResidentMaxRows;
    } else {
        rows = ((N + grid - 1) / grid + unit - 1) / unit * unit;
    }
    if (rows < unit) rows = unit;
    s.rows_per_wg = rows;
    const int chunks = (rows + 15) / 16;
    s.chunk_rows = whole16 ? 16 : (((rows + chunks - 1) / chunks + 3) & ~3);
    s.prefetch = prefetch;
    if (prefetch == 0) {
        s.prefetch = (chunks == 2 && M <= 8) ? 2 : 1;
        if (s.prefetch == 2 && !decode_resident_supported(M, N, K, s)) s.prefetch = 1;
    }
    if (!decode_resident_supported(M, N, K, s)) return false;
    *out = s;
    return true;
}

// Output tile of the LDS-staged kernel.  A launch runs in rounds of as many workgroups as the chip holds at once,
// so the estimate is rounds x tile area / relative efficiency of the tile shape (measured on LLaMA-13B shapes): the
// big tile does the most work per byte staged, the smaller ones fill the chip when N is small.
int choose_prefill_tile(int M, int N) {
    struct Option { int id, bm, bn, per_cu; double eff; };
    const Option options[] = {{kPrefillTile128x256, 128, 256, 2, 1.00},
                              {kPrefillDma128x160, 128, 160, 2, 0.80},  // the LDS-direct variant is the faster 128 x 160
                              {kPrefillTile128x128, 128, 128, 3, 0.78}};
    const int cus = compute_units();
    int best = kPrefillTile128x256;
    double best_cost = 0;
    for (const Option &o : options) {
        const long long tiles = (long long)((M + o.bm - 1) / o.bm) * ((N + o.bn - 1) / o.bn);
        const long long slots = (long long)cus * o.per_cu;
        const long long full = tiles / slots, rest = tiles % slots;
        // a partial last round costs at least half a round: its workgroups no longer share their compute unit
        const double rounds = (double)full + (rest == 0 ? 0.0 : (rest * 2 <= slots ? 0.5 : (double)rest / slots * 0.5 + 0.5));
        const double cost = rounds * o.bm * o.bn * o.per_cu / o.eff;
        if (best_cost == 0 || cost < best_cost) { best_cost = cost; best = o.id; }
    }
    return best;
}

// Output tile of the kernel over the tiled weight layout.  A launch runs in rounds of as many workgroups as the chip
// holds at once; the estimate is rounds x tile area x workgroups per compute unit / efficiency of the tile shape.
// Efficiencies and the cost of a round in which a compute unit holds one workgroup instead of two ("alone") are
// measured on LLaMA-13B shapes, M = 128 .. 4096 (warm weights, tiles timed in turn within one process):
//   256 x 256         one per compute unit, the most work per operand byte staged;
//   256 x 192         its narrower partner: fills one round where 256 x 256 would need two, or leave columns over;
//   128 x 256 8 waves one per compute unit (three-stage ring): half the tile in 59 % of the time of 256 x 256;
//   128 x 256 4 waves two per compute unit (two-stage ring); alone on a compute unit it takes 73 % of a shared round;
//   128 x 160, 128 x 128, 64 x 128   two per compute unit, for N or M too small for the above;
//   128 x 128 with the k halves of a stage on two wave sets, one per compute unit.
// For 256 x 256 the estimate also covers the launch in two phases (whole rounds of 256 x 256, the columns left over as
// one round of 256 x 192, see launch_tiled_in_phases).
// max_id: the highest tile id the weight format has (the unsigned storage lacks the tiles above kTiledTileMax).
int choose_tiled_tile(int M, int N, int max_id = kTiledTileMax4) {
    struct Option { int id, bm, bn, per_cu; double eff, alone; };
    const Option options[] = {{kTiled256x256, 256, 256, 1, 1.00, 1.0},    {kTiled256x192, 256, 192, 1, 0.97, 1.0},
                              {kTiled128x256, 128, 256, 2, 0.93, 0.73},   {kTiled128x256W8, 128, 256, 1, 0.85, 1.0},
                              {kTiled128x160, 128, 160, 2, 0.66, 0.63},   {kTiled128x128, 128, 128, 2, 0.75, 0.67},
                              {kTiled64x128, 64, 128, 2, 0.60, 0.75},     {kTiled128x128K2, 128, 128, 1, 0.60, 1.0}};
    const int cus = compute_units();
    // Medium M: when not even 128 x 128 tiles occupy three quarters of the compute units, run time is the length of
    // one workgroup's walk over K, and smaller tiles (more workgroups, each with a shorter stage) shorten it.
    auto count = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    if (M <= 32) return kTiled32x128;  // taller tiles would multiply rows that do not exist
    if (M <= 64 || count(128, 128) * 4 < (long long)cus * 3)
        return count(64, 128) * 4 >= (long long)cus * 3 ? kTiled64x128 : kTiled64x64;
    int best = kTiled256x256;
    double best_cost = 0;
    for (const Option &o : options) {
        if (o.id > max_id) continue;
        const long long tiles = count(o.bm, o.bn);
        const long long slots = (long long)cus * o.per_cu;
        const long long full = tiles / slots, rest = tiles % slots;
        const double last = rest == 0 ? 0.0 : ((o.per_cu > 1 && rest <= cus) ? o.alone : 1.0);
        double cost = ((double)full + last) * o.bm * o.bn * o.per_cu / o.eff;
        if (o.id == kTiled256x256 && max_id >= kTiled256x192) {
            const long long tiles_m = (M + 255) / 256, cols = (N + 255) / 256, per_round = cus / tiles_m;
            if (per_round > 0 && cols > per_round && cols % per_round != 0) {
                const long long rest_cols = N - (cols / per_round) * per_round * 256;
                const double phased = (double)(cols / per_round) * 256 * 256 + 256 * 192 / 0.97;
                if ((rest_cols + 191) / 192 <= per_round && phased < cost) cost = phased;
            }
        }
        if (best_cost == 0 || cost < best_cost) { best_cost = cost; best = o.id; }
    }
    return best;
}

// The choice among the fine-grained variant's tiles (measured on LLaMA-13B shapes at M = 1024 and 4096: two
// 128 x 128 workgroups per compute unit are never slower than one 128 x 256 workgroup of 8 waves).
int choose_fine_tile(int M, int N) {
    const int cus = compute_units();
    auto count = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    if (M <= 32) return kFine32x128;
    if (M <= 64 || count(128, 128) * 4 < (long long)cus * 3)
        return count(64, 128) * 4 >= (long long)cus * 3 ? kFine64x128 : kFine64x64;
    struct Option { int id, bm, bn, per_cu; double eff; };
    const Option options[] = {{kFine128x256, 128, 256, 1, 0.95}, {kFine128x128, 128, 128, 2, 1.00}};
    int best = kFine128x256;
    double best_cost = 0;
    for (const Option &o : options) {
        const long long tiles = count(o.bm, o.bn);
        const long long slots = (long long)cus * o.per_cu;
        const long long full = tiles / slots, rest = tiles % slots;
        const double last = rest == 0 ? 0.0 : (o.per_cu == 1 || rest * 2 > slots ? 1.0 : 0.5);
        const double cost = ((double)full + last) * o.bm * o.bn * o.per_cu / o.eff;
        if (best_cost == 0 || cost < best_cost) { best_cost = cost; best = o.id; }
    }
    return best;
}

// The same choice for the int8-weight variant, whose weight stages take twice the LDS (shallower rings, and the
// 128 x 256 tile fits a compute unit only once).
int choose_tiled_tile8(int M, int N) {
    const int cus = compute_units();
    auto count = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    if (M <= 32) return kTiled32x128;  // taller tiles would multiply rows that do not exist
    if (M <= 64 || count(128, 128) * 4 < (long long)cus * 3)
        return count(64, 128) * 4 >= (long long)cus * 3 ? kTiled64x128 : kTiled64x64;
    struct Option { int id, bm, bn, per_cu; double eff; };
    const Option options[] = {{kTiled256x256, 256, 256, 1, 1.00},
                              {kTiled128x256, 128, 256, 1, 0.80},
                              {kTiled128x160, 128, 160, 2, 0.95},
                              {kTiled128x128, 128, 128, 2, 0.85}};
    int best = kTiled256x256;
    double best_cost = 0;
    for (const Option &o : options) {
        const long long tiles = count(o.bm, o.bn);
        const long long slots = (long long)cus * o.per_cu;
        const long long full = tiles / slots, rest = tiles % slots;
        const double last = rest == 0 ? 0.0 : (o.per_cu == 1 || rest * 2 > slots ? 1.0 : 0.5);
        const double cost = ((double)full + last) * o.bm * o.bn * o.per_cu / o.eff;
        if (best_cost == 0 || cost < best_cost) { best_cost = cost; best = o.id; }
    }
    return best;
}

// Tiling choice.  Small M streams the weights once (HBM bound); large M goes to the LDS-staged tiling
// (matrix-core bound).  `variant` refines a forced tiling (see w4a8.h); 0 lets the library choose.
int choose_plan(int M, int N, int K, int tiling, int variant, Plan *pl) {
    pl->tiling = tiling;
    if (tiling == W4A8_TILING_AUTO_TILED) {
        // one weight array for every M: the weight-streaming kernels up to M = 16 and, where all of K fits a wave's
        // registers, up to M = 64; the large-M kernel above
        if (M > 16)
            pl->tiling = wide_plan(M, N, K, 1, 1, &pl->decode) ? W4A8_TILING_DECODE_RESIDENT_TILED : W4A8_TILING_PREFILL_TILED;
        else
            pl->tiling = (resident_shape(M, N, K, 0, 0, 0, false, -1, true, &pl->decode, 1, true) ||
                          resident_shape(M, N, K, 0, 0, 0, false, -1, true, &pl->decode))
                             ? W4A8_TILING_DECODE_RESIDENT_TILED
                             : W4A8_TILING_DECODE_STREAM_TILED;
    }
    const bool decode_tiled = pl->tiling == W4A8_TILING_DECODE_RESIDENT_TILED || pl->tiling == W4A8_TILING_DECODE_STREAM_TILED;
    if (pl->tiling == W4A8_TILING_DECODE_RESIDENT_TILED) pl->tiling = W4A8_TILING_DECODE_RESIDENT;
    if (pl->tiling == W4A8_TILING_DECODE_STREAM_TILED) pl->tiling = W4A8_TILING_DECODE_STREAM;
    if (tiling == W4A8_TILING_AUTO) {
        if (M > kDecodeMaxM)
            pl->tiling = W4A8_TILING_PREFILL;
        else
            pl->tiling = resident_shape(M, N, K, 0, 0, 0, false, -1, false, &pl->decode) ? W4A8_TILING_DECODE_RESIDENT
                                                                                          : W4A8_TILING_DECODE_STREAM;
    }
    if (pl->tiling == W4A8_TILING_DECODE_RESIDENT) {
        if (M > kResidentMaxM) return W4A8_ERR_ARG;
        const int flags = variant / 100000000, prefetch = variant / 10000000 % 10, waves = variant / 100000 % 100;
        // The library's own choice over the tiled array: per-wave staging from five tokens on (measured on LLaMA-13B
        // shapes: level with the whole-row staging at 5 or 6 tokens, 6 to 20 % faster at 16, where the whole rows crowd
        // or overflow LDS; below five tokens its extra round trip per window costs up to 8 % on a long K).
        const bool want_window = (flags & 16) != 0 || (tiling == W4A8_TILING_AUTO_TILED && M >= 5);
        auto shape = [&](bool window) {
            return resident_shape(M, N, K, waves, variant % 100000, prefetch, (flags & 1) != 0,
                                  (flags & 2) ? 2 : (flags & 8) ? 0 : -1, decode_tiled, &pl->decode, 1, window);
        };
        if (!(want_window && shape(true)) && !((flags & 16) == 0 && shape(false))) return W4A8_ERR_ARG;
        pl->decode.x_direct = (flags & 4) != 0;
    } else if (pl->tiling == W4A8_TILING_DECODE_STREAM) {
        if (M > kDecodeMaxM) return W4A8_ERR_ARG;
        const int mt = (M + 15) / 16;
        DecodeShape s{};
        s.resident = false;
        s.tiled = decode_tiled;
        // K beyond the resident kernel's reach at token-generation sizes (70B down, K = 28672): two row tiles on four
        // waves stream 7 % faster than the general default (measured, cold weights)
        const bool long_k_decode = mt == 1 && K > 16384;
        s.row_tiles = variant ? variant / 100 : ((M <= 8 && !long_k_decode) ? 1 : 2);
        s.waves = variant ? variant % 100 : (((mt >= 4 && s.row_tiles == 2) || long_k_decode) ? 4 : 8);
        if ((s.row_tiles != 1 && s.row_tiles != 2) || (s.waves != 4 && s.waves != 8)) return W4A8_ERR_ARG;
        if (mt == 4 && s.row_tiles == 2 && s.waves == 8) return W4A8_ERR_ARG;  // would not fit in LDS
        pl->decode = s;
    } else if (pl->tiling == W4A8_TILING_PREFILL_TILED) {
        if (variant < 0 || variant > kTiledTileMax4) return W4A8_ERR_ARG;
        pl->prefill_tile = variant ? variant : choose_tiled_tile(M, N);
    } else {
        if (variant < 0 || variant > kPrefillTileMax) return W4A8_ERR_ARG;
        pl->prefill_tile = variant ? variant : choose_prefill_tile(M, N);
    }
    return W4A8_OK;
}

// The library's own launch of the large-M kernel over tiled int4 weights.  Where 256 x 256 tiles fill the chip more
// than once, the last, partial round costs as much as a full one (LLaMA-13B gate+up at M = 1024: 432 tiles on 256
// compute units, i.e. two rounds for 1.69 rounds of work).  Then the columns that whole rounds cover go to one launch
// and the columns left over to a second launch with 256 x 192 tiles, if those fit into a single round: the second
// round shrinks to three quarters.  Two launches of the same kernel on disjoint column ranges of the same output:
// same arithmetic, same bits.
hipError_t launch_tiled_in_phases(const PrefillArgs &a, bool want_acc, int tile, hipStream_t st) {
    const int cus = compute_units();
    const long long tiles_m = (a.M + 255) / 256, cols = (a.N + 255) / 256;
    const long long per_round = tiles_m > 0 ? cus / tiles_m : 0;  // column tiles of 256 that one round holds
    if (tile != kTiled256x256 || per_round == 0 || cols <= per_round || cols % per_round == 0)
        return launch_gemm_prefill_tiled(a, want_acc, tile, st);
    const long long n_first = (cols / per_round) * per_round * 256;     // covered by whole rounds
    const long long rest = a.N - n_first;
    if ((rest + 191) / 192 > per_round) return launch_gemm_prefill_tiled(a, want_acc, tile, st);  // 192 wide would need two rounds too
    PrefillArgs first = a, second = a;
    first.N = (int)n_first;
    second.N = (int)rest;
    second.wp = a.wp + (size_t)(n_first / 32) * (size_t)((a.K + kTiledBlockK - 1) / kTiledBlockK) * (size_t)kTiledBlockBytes;
    if (a.s_w) second.s_w = a.s_w + n_first;
    if (a.out) second.out = (unsigned short *)a.out + n_first;
    if (a.acc_out) second.acc_out = a.acc_out + n_first;
    if (const hipError_t e = launch_gemm_prefill_tiled(first, want_acc, kTiled256x256, st); e != hipSuccess) return e;
    return launch_gemm_prefill_tiled(second, want_acc, kTiled256x192, st);
}

int run_gemm(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w, void *out_fp16, int32_t *acc_i32,
             int M, int N, int K, int tiling, int variant, void *stream) {
    const bool want_acc = acc_i32 != nullptr;
    if ((out_fp16 != nullptr) == want_acc) return W4A8_ERR_NULL;  // exactly one output
    if (!xq || !wp) return W4A8_ERR_NULL;
    if (!want_acc && (!s_a || !s_w)) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (tiling < W4A8_TILING_AUTO || tiling > W4A8_TILING_AUTO_TILED || variant < 0) return W4A8_ERR_ARG;
    if (misaligned(xq) || misaligned(wp) || misaligned(out_fp16) || misaligned(acc_i32) || (s_w && misaligned(s_w)))
        return W4A8_ERR_ALIGN;

    Plan pl{};
    if (int e = choose_plan(M, N, K, tiling, variant, &pl)) return e;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t err;
    if (pl.tiling == W4A8_TILING_PREFILL_TILED) {
        PrefillArgs a{};
        a.xq = xq; a.s_a = s_a; a.wp = wp; a.s_w = s_w;
        a.out = out_fp16; a.acc_out = acc_i32;
        a.M = M; a.N = N; a.K = K; a.ldc = N;
        err = variant == 0 ? launch_tiled_in_phases(a, want_acc, pl.prefill_tile, st)
                           : launch_gemm_prefill_tiled(a, want_acc, pl.prefill_tile, st);
    } else if (pl.tiling != W4A8_TILING_PREFILL) {
        DecodeArgs a{};
        a.xq = xq; a.s_a = s_a; a.wp = wp; a.s_w = s_w;
        a.out = out_fp16; a.acc_out = acc_i32;
        a.M = M; a.N = N; a.K = K;
        a.rows_per_wg = pl.decode.rows_per_wg;
        a.chunk_rows = pl.decode.chunk_rows;
        a.x_lds_pitch = pl.decode.x_direct ? -1 : 0;
        err = launch_gemm_decode(a, want_acc, pl.decode, st);
    } else {
        PrefillArgs a{};
        a.xq = xq; a.s_a = s_a; a.wp = wp; a.s_w = s_w;
        a.out = out_fp16; a.acc_out = acc_i32;
        a.M = M; a.N = N; a.K = K; a.ldc = N;
        err = launch_gemm_prefill(a, want_acc, pl.prefill_tile, st);
    }
    return launched(err);
}

}  // namespace

extern "C" {

int w4a8_version(void) { return 100; }

const char *w4a8_last_hip_error(void) { return hipGetErrorName(last_hip_error); }

const char *w4a8_strerror(int err) {
    switch (err) {
        case W4A8_OK: return "ok";
        case W4A8_ERR_NULL: return "a required pointer is NULL (or both / neither output given)";
        case W4A8_ERR_SHAPE: return "shape outside the contract: M,N >= 1, 32 <= K <= 65536, K % 32 == 0";
        case W4A8_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case W4A8_ERR_WORKSPACE: return "workspace smaller than w4a8_gemm_workspace_bytes reports";
        case W4A8_ERR_LAUNCH: return "HIP rejected the kernel launch";
        case W4A8_ERR_VALUE: return "weight code outside [-8, 7]";
        case W4A8_ERR_ARG: return "tiling id or variant not available for this shape";
        default: return "unknown w4a8 error code";
    }
}

int w4a8_quantize_act(const void *x_fp16, int8_t *xq, float *s_a, int M, int K, void *stream) {
    if (!x_fp16 || !xq || !s_a) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, 1, K)) return e;
    if (misaligned(x_fp16) || misaligned(xq)) return W4A8_ERR_ALIGN;
    return launched(launch_quantize_act(x_fp16, K, xq, s_a, M, K, static_cast<hipStream_t>(stream)));
}

int w4a8_quantize_act_strided(const void *x_fp16, long long ldx, int8_t *xq, float *s_a, int M, int K, void *stream) {
    if (!x_fp16 || !xq || !s_a) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, 1, K)) return e;
    if (ldx < K || (ldx & 7) != 0) return W4A8_ERR_SHAPE;  // rows must not overlap and must start 16-byte aligned
    if (misaligned(x_fp16) || misaligned(xq)) return W4A8_ERR_ALIGN;
    return launched(launch_quantize_act(x_fp16, ldx, xq, s_a, M, K, static_cast<hipStream_t>(stream)));
}

size_t w4a8_gemm_workspace_bytes(int M, int N, int K) {
    (void)M; (void)N; (void)K;
    return 0;  // no tiling needs scratch memory: partial sums meet in LDS
}

int w4a8_gemm(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w, void *out_fp16, int M, int N, int K,
              void *workspace, size_t workspace_bytes, void *stream) {
    (void)workspace; (void)workspace_bytes;
    if (!out_fp16) return W4A8_ERR_NULL;
    return run_gemm(xq, s_a, wp, s_w, out_fp16, nullptr, M, N, K, W4A8_TILING_AUTO, 0, stream);
}

int w4a8_gemm_acc_i32(const int8_t *xq, const uint8_t *wp, int32_t *acc, int M, int N, int K, void *workspace,
                      size_t workspace_bytes, void *stream) {
    (void)workspace; (void)workspace_bytes;
    if (!acc) return W4A8_ERR_NULL;
    return run_gemm(xq, nullptr, wp, nullptr, nullptr, acc, M, N, K, W4A8_TILING_AUTO, 0, stream);
}

int w4a8_gemm_tuned(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w, void *out_fp16,
                    int32_t *acc_i32, int M, int N, int K, int tiling, int variant, void *workspace, size_t workspace_bytes,
                    void *stream) {
    (void)workspace; (void)workspace_bytes;
    return run_gemm(xq, s_a, wp, s_w, out_fp16, acc_i32, M, N, K, tiling, variant, stream);
}

size_t w4a8_tiled_weight_bytes(int N, int K) {
    if (check_gemm_shape(1, N, K)) return 0;
    return tiled_weight_bytes(N, K);
}

int w4a8_tile_weights(const uint8_t *wp, uint8_t *wt, int N, int K, void *stream) {
    if (!wp || !wt) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(1, N, K)) return e;
    if (misaligned(wp) || misaligned(wt)) return W4A8_ERR_ALIGN;
    return launched(launch_tile_weights(wp, wt, N, K, static_cast<hipStream_t>(stream)));
}

int w4a8_gemm_tiled(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16, int M, int N,
                    int K, void *stream) {
    if (!out_fp16) return W4A8_ERR_NULL;
    return run_gemm(xq, s_a, wt, s_w, out_fp16, nullptr, M, N, K, W4A8_TILING_AUTO_TILED, 0, stream);
}

int w4a8_gemm_tiled_swiglu(const int8_t *xq, const float *s_a, const uint8_t *wt_gu, const float *s_w_gu, void *h_fp16, int M,
                           int I, int K, void *stream) {
    if (!xq || !s_a || !wt_gu || !s_w_gu || !h_fp16) return W4A8_ERR_NULL;
    if (I < 32 || (I % 32) != 0 || I > W4A8_MAX_K) return W4A8_ERR_SHAPE;  // I follows the K contract, as in w4a8_silu_mul
    const int N = 2 * I;
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (misaligned(xq) || misaligned(wt_gu) || misaligned(h_fp16) || misaligned(s_w_gu)) return W4A8_ERR_ALIGN;
    if ((long long)M * K > 0xF0000000ll || (long long)tiled_weight_bytes(N, K, 4) > 0xF0000000ll) return W4A8_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // up to 64 tokens: the weight-streaming kernel with per-wave staging, where it has a shape for (M, N, K)
    if (M <= kResidentMaxM) {
        DecodeShape shape{};
        shape.swiglu = true;
        if (resident_shape(M, N, K, 0, 0, 0, false, -1, true, &shape, 1, true)) {
            DecodeArgs d{};
            d.xq = xq; d.s_a = s_a; d.wp = wt_gu; d.s_w = s_w_gu; d.out = h_fp16;
            d.M = M; d.N = N; d.K = K;
            d.rows_per_wg = shape.rows_per_wg;
            d.chunk_rows = shape.chunk_rows;
            return launched(launch_gemm_decode(d, false, shape, st));
        }
    }
    int tile = choose_tiled_tile(M, N);
    if (tile != kTiled256x256 && tile != kTiled256x192 && tile != kTiled128x256 && tile != kTiled128x256W8)
        tile = kTiled128x128;  // the large-M kernel has the fused form for these tiles
    PrefillArgs a{};
    a.xq = xq; a.s_a = s_a; a.wp = wt_gu; a.s_w = s_w_gu; a.out = h_fp16;
    a.M = M; a.N = N; a.K = K; a.ldc = I;
    // the two-phase launch of launch_tiled_in_phases, with the output offset counted in values of h
    const int cus = compute_units();
    const long long tiles_m = (M + 255) / 256, cols = (N + 255) / 256, per_round = cus / tiles_m;
    if (tile == kTiled256x256 && per_round > 0 && cols > per_round && cols % per_round != 0) {
        const long long n_first = (cols / per_round) * per_round * 256, rest = N - n_first;
        if ((rest + 191) / 192 <= per_round) {
            PrefillArgs first = a, second = a;
            first.N = (int)n_first;
            second.N = (int)rest;
            second.wp = wt_gu + (size_t)(n_first / 32) * (size_t)((K + kTiledBlockK - 1) / kTiledBlockK) * (size_t)kTiledBlockBytes;
            second.s_w = s_w_gu + n_first;
            second.out = (unsigned short *)h_fp16 + n_first / 2;
            if (int e = launched(launch_gemm_prefill_tiled_swiglu(first, kTiled256x256, st))) return e;
            return launched(launch_gemm_prefill_tiled_swiglu(second, kTiled256x192, st));
        }
    }
    return launched(launch_gemm_prefill_tiled_swiglu(a, tile, st));
}

// ---- K split over workgroups for shapes whose tiles alone leave most of the chip idle (medium M, small N)

namespace {

struct SplitPlan { int tile, splits, stages_per_split; };

// Tile and number of K slices (measured on LLaMA-13B shapes, M = 32 .. 512).  Slices pay where the tiles alone leave
// the chip under-filled: up to half the compute units for a short walk over K (fewer than 64 stages), up to all of
// them for a long one; they aim at two workgroups per compute unit, at least 12 stages per slice and at most 6 slices
// (each slice adds a slab to write and to read again).  With slices available the 64 x 128 tile replaces the
// 64 x 64 one, and the 128 x 128 tile the 64 x 128 one on a long K (same workgroup count after the split, fewer operand
// bytes per MFMA).  M above 512 is left alone: there the tiles fill the chip or the slabs cost more than they save.
SplitPlan plan_split(int M, int N, int K, int variant, int splits) {
    SplitPlan pl{};
    const int st_all = (K + kTiledBlockK - 1) / kTiledBlockK;
    const int cus = compute_units();
    const bool long_k = st_all >= 64;
    auto count = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    pl.tile = variant ? variant : choose_tiled_tile(M, N);
    const int unsplit_tile = pl.tile;
    if (!variant && M > 64 && M <= 512) {
        if (pl.tile == kTiled64x64) pl.tile = kTiled64x128;
        if (long_k && pl.tile == kTiled64x128 && count(128, 128) <= cus) pl.tile = kTiled128x128;
    }
    int s = splits;
    if (s == 0) {
        static const int bm[] = {0, 256, 256, 128, 128, 128, 64, 64, 32, 128, 128, 256, 128};
        static const int bn[] = {0, 256, 256, 256, 160, 128, 128, 64, 128, 160, 128, 192, 256};
        const long long tiles = count(bm[pl.tile], bn[pl.tile]);
        s = 1;
        if (M <= 512 && tiles <= (long_k ? cus : cus / 2)) {
            s = (int)((2 * (long long)cus + tiles / 2) / tiles);
            if (s > 6) s = 6;
            if (s > st_all / 12) s = st_all / 12;
            if (s < 1) s = 1;
        }
    }
    if (s > st_all) s = st_all;
    if (s <= 1) pl.tile = unsplit_tile;  // the larger tiles are only worth it together with the slices
    pl.stages_per_split = (st_all + s - 1) / s;
    pl.splits = (st_all + pl.stages_per_split - 1) / pl.stages_per_split;  // no empty slice
    return pl;
}

// What w4a8_gemm_tiled_splitk does with a shape.  Up to 16 tokens (no tile or slice count forced): the weight-streaming
// kernels, no slabs.  17 to 64 tokens (no tile forced): the persistent kernel with per-wave staging, in as few K slices
// as a wave's registers allow (or the forced count, if an instantiation exists for it).  Otherwise the LDS-staged
// kernel with the slices of plan_split.
struct SplitRoute {
    enum Kind { kStream, kWide, kRing } kind;
    DecodeShape wide;
    SplitPlan ring;
    size_t slab_bytes;  // workspace the route needs
};

SplitRoute split_route(int M, int N, int K, int variant, int splits) {
    SplitRoute r{};
    const size_t slab = (size_t)M * (size_t)N * sizeof(int32_t);
    if (M <= 16 && variant == 0 && splits == 0) {
        r.kind = SplitRoute::kStream;
    } else if (variant == 0 && wide_plan(M, N, K, splits, 8, &r.wide)) {
        r.kind = SplitRoute::kWide;
        r.slab_bytes = r.wide.k_slices > 1 ? (size_t)r.wide.k_slices * slab : 0;
    } else {
        r.kind = SplitRoute::kRing;
        r.ring = plan_split(M, N, K, variant, splits);
        r.slab_bytes = r.ring.splits > 1 ? (size_t)r.ring.splits * slab : 0;
    }
    return r;
}

}  // namespace

size_t w4a8_gemm_tiled_workspace_bytes(int M, int N, int K) {
    if (check_gemm_shape(M, N, K)) return 0;
    // the library's own choice never exceeds 8 slices; a forced count is checked against the buffer at the call
    return split_route(M, N, K, 0, 0).slab_bytes;
}

int w4a8_gemm_tiled_splitk(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16, int M,
                           int N, int K, int variant, int splits, void *workspace, size_t workspace_bytes, void *stream) {
    if (!xq || !s_a || !wt || !s_w || !out_fp16) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (variant < 0 || variant > kTiledTileMax4 || splits < 0 || splits > 64) return W4A8_ERR_ARG;
    if (misaligned(xq) || misaligned(wt) || misaligned(out_fp16) || misaligned(s_w) || misaligned(workspace))
        return W4A8_ERR_ALIGN;
    const SplitRoute route = split_route(M, N, K, variant, splits);
    if (route.kind == SplitRoute::kStream)  // token generation: the weight-streaming kernels over the same array
        return run_gemm(xq, s_a, wt, s_w, out_fp16, nullptr, M, N, K, W4A8_TILING_AUTO_TILED, 0, stream);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (route.kind == SplitRoute::kWide) {
        const DecodeShape &ds = route.wide;
        DecodeArgs d{};
        d.xq = xq; d.s_a = s_a; d.wp = wt; d.s_w = s_w;
        d.M = M; d.N = N; d.K = K;
        d.rows_per_wg = ds.rows_per_wg;
        d.chunk_rows = ds.chunk_rows;
        if (ds.k_slices <= 1) {
            d.out = out_fp16;
            return launched(launch_gemm_decode(d, false, ds, st));
        }
        if (!workspace) return W4A8_ERR_NULL;
        if (workspace_bytes < route.slab_bytes) return W4A8_ERR_WORKSPACE;
        d.acc_out = static_cast<int32_t *>(workspace);
        if (int e = launched(launch_gemm_decode(d, true, ds, st))) return e;
        return launched(launch_splitk_epilogue(d.acc_out, ds.k_slices, s_a, s_w, out_fp16, M, N, st));
    }
    const SplitPlan pl = route.ring;
    PrefillArgs a{};
    a.xq = xq; a.s_a = s_a; a.wp = wt; a.s_w = s_w;
    a.M = M; a.N = N; a.K = K; a.ldc = N;
    if (pl.splits <= 1) {
        a.out = out_fp16;
        const hipError_t e = variant == 0 ? launch_tiled_in_phases(a, false, pl.tile, st)
                                          : launch_gemm_prefill_tiled(a, false, pl.tile, st);
        return launched(e);
    }
    // one launch must cover the problem (slabs are whole M x N matrices)
    if ((long long)M * K > 0xF0000000ll || (long long)tiled_weight_bytes(N, K, 4) > 0xF0000000ll) return W4A8_ERR_SHAPE;
    if (!workspace) return W4A8_ERR_NULL;
    if (workspace_bytes < (size_t)pl.splits * (size_t)M * (size_t)N * sizeof(int32_t)) return W4A8_ERR_WORKSPACE;
    a.acc_out = static_cast<int32_t *>(workspace);
    a.splits = pl.splits;
    a.stages_per_split = pl.stages_per_split;
    if (int e = launched(launch_gemm_prefill_tiled(a, true, pl.tile, st))) return e;
    return launched(launch_splitk_epilogue(a.acc_out, pl.splits, s_a, s_w, out_fp16, M, N, st));
}

// what the norm in front of the fused quantiser needs (gamma == NULL: no norm)
struct NormArgs {
    const void *res;
    long long ldres;
    const void *gamma;
    float eps;
    void *r_out, *y_out;
};

// quantiser + GEMM in one launch; swiglu: N = 2 I interleaved gate / up channels, out = h
static int linear_tiled(const void *x_fp16, long long ldx, const uint8_t *wt, const float *s_w, void *out_fp16, float *s_a_out,
                        int M, int N, int K, bool swiglu, void *stream, const NormArgs *norm = nullptr) {
    if (!x_fp16 || !wt || !s_w || !out_fp16) return W4A8_ERR_NULL;
    if (norm) {
        if (!norm->gamma) return W4A8_ERR_NULL;
        if (!(norm->eps >= 0.0f) || !(norm->eps < 3.0e38f)) return W4A8_ERR_ARG;
        if (norm->res && (norm->ldres < K || (norm->ldres & 7) != 0)) return W4A8_ERR_SHAPE;
        if (misaligned(norm->res) || misaligned(norm->gamma) || misaligned(norm->r_out) || misaligned(norm->y_out)) return W4A8_ERR_ALIGN;
        if (norm->res && ((unsigned long long)(M > 0 ? M - 1 : 0) * (unsigned long long)norm->ldres + (unsigned long long)K) * 2ull > 0xFFFF0000ull)
            return W4A8_ERR_SHAPE;
    }
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (ldx < K || (ldx & 7) != 0) return W4A8_ERR_SHAPE;  // rows must not overlap and must start 16-byte aligned
    if (misaligned(x_fp16) || misaligned(wt) || misaligned(out_fp16) || misaligned(s_w)) return W4A8_ERR_ALIGN;
    if (M > 4) return W4A8_ERR_ARG;
    if (((unsigned long long)(M - 1) * (unsigned long long)ldx + (unsigned long long)K) * 2ull > 0xFFFF0000ull) return W4A8_ERR_SHAPE;
    DecodeShape shape{};
    shape.fused_quant = true;
    shape.swiglu = swiglu;
    shape.norm = norm != nullptr;
    if (!resident_shape(M, N, K, 0, 0, 0, false, -1, true, &shape)) return W4A8_ERR_ARG;
    // both copies of the rows (fp16 and int8, padded to the 1 KB pieces of the copy; with the norm the residual rows as
    // well) must fit in LDS beside the slots of the partial sums
    const long long row_bytes = ((K + 1023) / 1024) * 1024 + 16 + (norm ? 2 : 1) * ((2ll * K + 1023) / 1024) * 1024;
    if (row_bytes * M + 3 * 1024 + 2ll * shape.prefetch * shape.waves * 1024 > 160 * 1024) return W4A8_ERR_ARG;
    DecodeArgs a{};
    a.x16 = static_cast<const uint16_t *>(x_fp16);
    a.ldx = ldx;
    a.s_a_out = s_a_out;
    a.wp = wt; a.s_w = s_w; a.out = out_fp16;
    a.M = M; a.N = N; a.K = K;
    a.rows_per_wg = shape.rows_per_wg;
    a.chunk_rows = shape.chunk_rows;
    if (norm) {
        a.res16 = static_cast<const uint16_t *>(norm->res);
        a.ldres = norm->ldres;
        a.gamma = static_cast<const uint16_t *>(norm->gamma);
        a.eps = norm->eps;
        a.r_out = static_cast<uint16_t *>(norm->r_out);
        a.y_out = static_cast<uint16_t *>(norm->y_out);
    }
    return launched(launch_gemm_decode(a, false, shape, static_cast<hipStream_t>(stream)));
}

int w4a8_linear_tiled_norm_fp16(const void *x_fp16, long long ldx, const void *res_fp16, long long ldres, const void *gamma_fp16,
                                float eps, void *r_out_fp16, void *y_out_fp16, const uint8_t *wt, const float *s_w, void *out_fp16,
                                float *s_a_out, int M, int N, int K, int swiglu, void *stream) {
    if (swiglu != 0 && swiglu != 1) return W4A8_ERR_ARG;
    if (swiglu && ((N & 63) != 0 || N / 2 > W4A8_MAX_K)) return W4A8_ERR_SHAPE;  // N = 2 I, I follows the K contract
    const NormArgs norm{res_fp16, ldres, gamma_fp16, eps, r_out_fp16, y_out_fp16};
    return linear_tiled(x_fp16, ldx, wt, s_w, out_fp16, s_a_out, M, N, K, swiglu != 0, stream, &norm);
}

int w4a8_linear_tiled_fp16(const void *x_fp16, long long ldx, const uint8_t *wt, const float *s_w, void *out_fp16,
                           float *s_a_out, int M, int N, int K, void *stream) {
    return linear_tiled(x_fp16, ldx, wt, s_w, out_fp16, s_a_out, M, N, K, false, stream);
}

int w4a8_linear_tiled_swiglu_fp16(const void *x_fp16, long long ldx, const uint8_t *wt_gu, const float *s_w_gu, void *h_fp16,
                                  float *s_a_out, int M, int I, int K, void *stream) {
    if (I < 32 || (I % 32) != 0 || I > W4A8_MAX_K) return W4A8_ERR_SHAPE;
    return linear_tiled(x_fp16, ldx, wt_gu, s_w_gu, h_fp16, s_a_out, M, 2 * I, K, true, stream);
}

int w4a8_gemm_tiled_splitk_static(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16,
                                  int M, int N, int K, int variant, int splits, void *stream) {
    if (!xq || !s_a || !wt || !s_w || !out_fp16) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (variant < 0 || variant > kTiledTileMax4 || splits < 0 || splits > 64) return W4A8_ERR_ARG;
    if (split_route(M, N, K, variant, splits).slab_bytes > kStaticScratchBytes) return W4A8_ERR_WORKSPACE;
    void *ws = nullptr;
    if (int e = static_scratch(&ws)) return e;
    return w4a8_gemm_tiled_splitk(xq, s_a, wt, s_w, out_fp16, M, N, K, variant, splits, ws, kStaticScratchBytes, stream);
}

int w4a8_init(void) {
    void *ws = nullptr;
    if (int e = static_scratch(&ws)) return e;
    (void)compute_units();
    if (int e = launched(prepare_tiled_kernels())) return e;
    return launched(prepare_decode_kernels());
}

// ---- W8A8 comparison variant: int8 weight codes in the tiled layout, the same kernels without the int4 conversion

size_t w8a8_tiled_weight_bytes(int N, int K) {
    if (check_gemm_shape(1, N, K)) return 0;
    return tiled_weight_bytes(N, K, 8);
}

int w8a8_tile_weights(const int8_t *w8, uint8_t *wt, int N, int K, void *stream) {
    if (!w8 || !wt) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(1, N, K)) return e;
    if (misaligned(w8) || misaligned(wt)) return W4A8_ERR_ALIGN;
    return launched(launch_tile_weights8(w8, wt, N, K, static_cast<hipStream_t>(stream)));
}

static int gemm_tiled_variant(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16,
                              int32_t *acc_i32, int M, int N, int K, int variant, void *stream, int wfmt);

int w8a8_gemm_tiled(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16,
                    int32_t *acc_i32, int M, int N, int K, int variant, void *stream) {
    return gemm_tiled_variant(xq, s_a, wt, s_w, out_fp16, acc_i32, M, N, K, variant, stream, 8);
}

// ---- ablation: the vanilla unsigned storage (u = w + 8 in the nibbles, 8 subtracted in registers), same tiled layout

int w4a8_gemm_tiled_unsigned(const int8_t *xq, const float *s_a, const uint8_t *ut, const float *s_w, void *out_fp16,
                             int32_t *acc_i32, int M, int N, int K, int variant, void *stream) {
    return gemm_tiled_variant(xq, s_a, ut, s_w, out_fp16, acc_i32, M, N, K, variant, stream, kWeightsUnsigned4);
}

// ---- ablation: fine-grained (group-wise) weight scales, Eq. (5)

int w4a8_gemm_fine_grained(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_g, int ldg, void *out_fp16,
                           int M, int N, int K, int variant, void *stream) {
    if (!xq || !s_a || !wt || !s_g || !out_fp16) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (K % kTiledBlockK != 0 || ldg < N || (ldg & 3) != 0) return W4A8_ERR_SHAPE;
    // one launch covers the problem: every byte offset inside the kernel stays below 2^32
    const long long kMaxBytes = 0xF0000000ll;
    if ((long long)M * K > kMaxBytes || (long long)tiled_weight_bytes(N, K, 4) > kMaxBytes ||
        (long long)(K / kTiledBlockK) * ldg * 4 > kMaxBytes)
        return W4A8_ERR_SHAPE;
    if (variant < 0 || variant > kFineTileMax) return W4A8_ERR_ARG;
    if (misaligned(xq) || misaligned(wt) || misaligned(out_fp16) || misaligned(s_g)) return W4A8_ERR_ALIGN;
    PrefillArgs a{};
    a.xq = xq; a.s_a = s_a; a.wp = wt; a.s_w = s_g;
    a.out = out_fp16;
    a.M = M; a.N = N; a.K = K; a.ldc = N; a.ldg = ldg;
    const int tile = variant ? variant : choose_fine_tile(M, N);
    return launched(launch_gemm_prefill_tiled(a, false, tile, static_cast<hipStream_t>(stream), kWeightsFineGrained4));
}

static int gemm_tiled_variant(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16,
                              int32_t *acc_i32, int M, int N, int K, int variant, void *stream, int wfmt) {
    const bool want_acc = acc_i32 != nullptr;
    if ((out_fp16 != nullptr) == want_acc) return W4A8_ERR_NULL;  // exactly one output
    if (!xq || !wt) return W4A8_ERR_NULL;
    if (!want_acc && (!s_a || !s_w)) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (variant < 0 || variant > (wfmt == 4 ? kTiledTileMax4 : kTiledTileMax)) return W4A8_ERR_ARG;
    if (misaligned(xq) || misaligned(wt) || misaligned(out_fp16) || misaligned(acc_i32) || (s_w && misaligned(s_w)))
        return W4A8_ERR_ALIGN;
    PrefillArgs a{};
    a.xq = xq; a.s_a = s_a; a.wp = wt; a.s_w = s_w;
    a.out = out_fp16; a.acc_out = acc_i32;
    a.M = M; a.N = N; a.K = K; a.ldc = N;
    const int tile = variant ? variant
                             : wfmt == 8 ? choose_tiled_tile8(M, N)
                                         : choose_tiled_tile(M, N, wfmt == 4 ? kTiledTileMax4 : kTiledTileMax);
    return launched(launch_gemm_prefill_tiled(a, want_acc, tile, static_cast<hipStream_t>(stream), wfmt));
}

int w4a8_quantize_weights(const void *w_fp16, uint8_t *wp, float *s_w, int N, int K, void *stream) {
    if (!w_fp16 || !wp || !s_w) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(1, N, K)) return e;
    if (misaligned(w_fp16) || misaligned(wp)) return W4A8_ERR_ALIGN;
    return launched(launch_quantize_weights(w_fp16, wp, s_w, N, K, static_cast<hipStream_t>(stream)));
}

int w4a8_quantize_weights_clipped(const void *w_fp16, const float *gamma, const float *beta, uint8_t *wp, float *s_w, int N,
                                  int K, void *stream) {
    if (!w_fp16 || !wp || !s_w) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(1, N, K)) return e;
    if (misaligned(w_fp16) || misaligned(wp)) return W4A8_ERR_ALIGN;
    return launched(launch_quantize_weights_clip(w_fp16, gamma, beta, wp, s_w, N, K, static_cast<hipStream_t>(stream)));
}

int w4a8_silu_mul(const void *gate_up_fp16, void *h_fp16, int M, int I, void *stream) {
    if (!gate_up_fp16 || !h_fp16) return W4A8_ERR_NULL;
    if (M < 1 || I < 8 || (I % 8) != 0 || M > 65535) return W4A8_ERR_SHAPE;
    if (misaligned(gate_up_fp16) || misaligned(h_fp16)) return W4A8_ERR_ALIGN;
    return launched(launch_silu_mul(gate_up_fp16, h_fp16, M, I, static_cast<hipStream_t>(stream)));
}

int w4a8_silu_mul_quantize(const void *gate_up_fp16, int8_t *xq, float *s_a, int M, int I, void *stream) {
    if (!gate_up_fp16 || !xq || !s_a) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, 1, I)) return e;  // I is the K of the GEMM that consumes xq
    if (misaligned(gate_up_fp16) || misaligned(xq)) return W4A8_ERR_ALIGN;
    return launched(launch_silu_mul_quantize(gate_up_fp16, xq, s_a, M, I, static_cast<hipStream_t>(stream)));
}

// ---- probes of what the chip sustains (context for the measurements, no part of the path)

int w4a8_add_rmsnorm_quantize(const void *x_fp16, const void *res_fp16, const void *gamma_fp16, float eps, void *r_out_fp16,
                              void *y_out_fp16, int8_t *xq, float *s_a, int M, int K, void *stream) {
    if (!x_fp16 || !gamma_fp16 || !xq || !s_a) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, 1, K)) return e;
    if (!(eps >= 0.0f) || !(eps < 3.0e38f)) return W4A8_ERR_ARG;  // also refuses NaN
    if (misaligned(x_fp16) || misaligned(res_fp16) || misaligned(gamma_fp16) || misaligned(r_out_fp16) || misaligned(y_out_fp16) ||
        misaligned(xq))
        return W4A8_ERR_ALIGN;
    return launched(launch_add_rmsnorm_quantize(x_fp16, res_fp16, gamma_fp16, eps, r_out_fp16, y_out_fp16, xq, s_a, M, K,
                                                static_cast<hipStream_t>(stream)));
}

int w4a8_probe_stream_read(const void *buf, size_t bytes, void *sink, void *stream) {
    if (!buf || !sink) return W4A8_ERR_NULL;
    if (bytes < 16) return W4A8_ERR_SHAPE;
    if (misaligned(buf)) return W4A8_ERR_ALIGN;
    return launched(launch_probe_stream_read(buf, bytes, static_cast<unsigned *>(sink), 8 * compute_units(), static_cast<hipStream_t>(stream)));
}

int w4a8_probe_read_pattern(const void *buf, size_t bytes, void *sink, int pattern, int loads, int workgroups_per_cu,
                            void *stream) {
    if (!buf || !sink) return W4A8_ERR_NULL;
    if (bytes < 16 || bytes > 0xFFFFFFF0ull) return W4A8_ERR_SHAPE;
    if (misaligned(buf)) return W4A8_ERR_ALIGN;
    if (pattern < 0 || pattern > 5 || (loads != 4 && loads != 8 && loads != 16) || workgroups_per_cu < 1 || workgroups_per_cu > 64)
        return W4A8_ERR_ARG;
    return launched(launch_probe_read_pattern(buf, bytes, static_cast<unsigned *>(sink), pattern, loads, workgroups_per_cu * compute_units(), static_cast<hipStream_t>(stream)));
}

int w4a8_probe_mixed_read(const void *cold, size_t cold_bytes, const void *hot, size_t hot_bytes, void *sink, int mode,
                          void *stream) {
    if (!cold || !hot || !sink) return W4A8_ERR_NULL;
    if (misaligned(cold) || misaligned(hot)) return W4A8_ERR_ALIGN;
    if (mode < 0 || mode > 3) return W4A8_ERR_ARG;
    const int cus = compute_units();
    const size_t per_iter = (mode == 2 ? 4096u : 2048u) * 16u;               // cold bytes a workgroup reads per iteration
    if (hot_bytes < 16 || hot_bytes > 0xFFFFFFF0ull || cold_bytes < per_iter * (size_t)cus) return W4A8_ERR_SHAPE;
    size_t per_wg = cold_bytes / (size_t)cus / per_iter * per_iter;           // whole iterations, within the buffer
    if (per_wg > 0x0FFFFFF0ull) per_wg = 0x0FFFFFF0ull / per_iter * per_iter;
    return launched(launch_probe_mixed_read(cold, (unsigned)(per_wg / 16), hot, (unsigned)(hot_bytes / 16), static_cast<unsigned *>(sink),
                                            mode, cus, static_cast<hipStream_t>(stream)));
}

int w4a8_probe_mfma_int8(void *sink, int iters, int pattern, void *stream) {
    if (!sink) return W4A8_ERR_NULL;
    if (iters < 1 || iters > (1 << 24) || pattern < 0 || pattern > 1) return W4A8_ERR_ARG;
    return launched(launch_probe_mfma_i8(static_cast<int *>(sink), 2 * compute_units(), iters, pattern, static_cast<hipStream_t>(stream)));
}

int w4a8_pack_weights_host(const int8_t *wq_host, uint8_t *wp_host, int N, int K) {
    if (!wq_host || !wp_host) return W4A8_ERR_NULL;
    if (N < 1 || K < 2 || (K & 1)) return W4A8_ERR_SHAPE;
    const size_t total = (size_t)N * (size_t)(K / 2);
    for (size_t i = 0; i < total; ++i) {
        const int even = wq_host[2 * i], odd = wq_host[2 * i + 1];
        if (even < -8 || even > 7 || odd < -8 || odd > 7) return W4A8_ERR_VALUE;
    }
    for (size_t i = 0; i < total; ++i) {
        const unsigned even = (unsigned)wq_host[2 * i] & 15u, odd = (unsigned)wq_host[2 * i + 1] & 15u;
        wp_host[i] = (uint8_t)(even | (odd << 4));
    }
    return W4A8_OK;
}

}  // extern "C"
