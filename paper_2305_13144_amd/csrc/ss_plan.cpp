// Which kernel runs a projection, and in which launch shape (host arithmetic only).
#include "ss_plan.h"

#include <algorithm>
#include <atomic>

namespace ss {

namespace {
std::atomic<int> g_gemm_mode{0};
std::atomic<int> g_sweep_split{1};
std::atomic<int> g_tall_tiles{1};
constexpr int kSmallMaxKsplit = 8;   // sweep and skinny kernels: at most 8 k-slices
constexpr int kTiledMaxKsplit = 4;   // tiled kernel: at most 4
constexpr int kTiledNoSliceTiles = 256;  // from this many tiles on (one per compute unit) the tiled kernel runs unsliced
constexpr int kTiledFullGroups = 320;    // below that, k-slices double until it has this many workgroups
}

void set_gemm_mode(int mode)
{
    // bit 2 (value 4) added to a mode: the sweep kernel never splits a unit between two waves (A/B measurements)
    g_sweep_split.store((mode & 4) ? 0 : 1, std::memory_order_relaxed);
    // bit 3 (value 8): the tiled kernel never uses 128-row tiles (A/B measurements)
    g_tall_tiles.store((mode & 8) ? 0 : 1, std::memory_order_relaxed);
    g_gemm_mode.store(mode & 3, std::memory_order_relaxed);
}
int gemm_mode() { return g_gemm_mode.load(std::memory_order_relaxed); }

// Launch shape of a projection.
// Sweep kernel (<= 256 rows, at least 160 KiB of weights per compute unit and row strip; below that the launch is
// too short to amortise its start-up and the skinny kernel's finer split wins: measured at 16 rows, the 7B o
// projection, 131 KiB per unit, is 12 % faster in the skinny kernel, the 13B one, 205 KiB, 30 % faster here): one workgroup per compute unit and
// k-slice, a wave per output strip (per gate/up strip pair with the SwiGLU epilogue).  k-slices double
// until every workgroup has 4 or more waves of work, as far as the epilogue allows them, never below 16
// k-blocks per slice; a workgroup has 4 or 8 waves, and when 8 are not enough there are more workgroups.
// Skinny kernel (<= 64 rows otherwise), from sweeps on the 7B shapes: aim at 512+ workgroups; 4 strips per
// workgroup halve the activation re-reads and win when k is short, 2 strips when k is long or when the
// epilogue forbids k-slices (SwiGLU, logits); k-slices double until there are 512 workgroups, at most 8,
// never leaving a wave fewer than 4 k-blocks.  Tiled kernel: ksplit fills the chip when there are few
// 64x256 tiles.

// Strips per wave of the sweep kernel: a gate/up pair for the SwiGLU epilogue, otherwise one.  One strip per wave gives
// twice the units of two, so half the k-slices (longer sweeps, half the partial sums).  Two strips per wave halve the LDS
// operand reads per weight byte and were the better choice from 49 rows on while an activation was two operands; with
// one operand per activation they never are.  Same GPU, 7B shapes, decode step at context 100, one / two strips per wave:
// 64 rows 3.99 / 4.27 ms, 80 rows 4.36 / 4.58, 96 rows 4.82 / 5.04, 128 rows 5.59 / 5.81.
int sweep_nbw(int epilogue, int /*m_rows*/) { return epilogue == EPI_SWIGLU ? 2 : 1; }

GemmPlan gemm_plan(int N, int Kp, int m_rows, int epilogue, int n_cu, int max_ksplit)
{
    GemmPlan p{1, 2, 4, 1, 0, 0, 1, 4};
    const int KB = Kp / 32;
    const int mode = gemm_mode();
    if (m_rows <= kSweepMaxRows) {
        const size_t w_per_cu = (size_t)N * (size_t)Kp * 2 / (size_t)n_cu;
        const size_t mt_rows = (size_t)(m_rows + 15) / 16;   // activation re-reads grow with the row strips: sweep earlier
        if (mode == 2 || (mode == 0 && w_per_cu * mt_rows >= ((size_t)160 << 10))) {
            if (epilogue == EPI_SWIGLU) max_ksplit = 1;   // fused epilogue: no k-slices
            const int nbw = sweep_nbw(epilogue, m_rows);
            const int units = (N / 16 + nbw - 1) / nbw;
            while (units * p.ksplit < 4 * n_cu && p.ksplit * 2 <= max_ksplit && p.ksplit < kSmallMaxKsplit &&
                   KB / (p.ksplit * 2) >= 16)
                p.ksplit *= 2;
            int gn = std::max(1, std::min(units, n_cu / p.ksplit));
            if ((units + gn - 1) / gn > 8) gn = (units + 7) / 8;
            p.sweep_p = (units + gn - 1) / gn <= 4 ? 4 : 8;
            p.sweep_gn = gn;
            // above 96 rows a workgroup with at most 4 units runs 8 waves, two per unit: the work per weight byte
            // grows with the row strips and 4 waves (one per SIMD) stop keeping up with the weight stream (same GPU,
            // split / not split: 104 rows 5.09 / 5.18 ms per step, 112 rows 5.21 / 5.28, 128 rows 5.59 / 5.81; up to
            // 96 rows the two are equal to within 0.1 %)
            p.sweep_kh = (p.sweep_p == 4 && m_rows > 96 && g_sweep_split.load(std::memory_order_relaxed)) ? 2 : 1;
            return p;
        }
    }
    if (m_rows <= 64) {
        if (epilogue == EPI_SWIGLU) max_ksplit = 1;   // fused epilogue: no k-slices
        const int mt = (m_rows + 15) / 16;
        p.kd = mt == 1 ? 4 : 2;
        if (max_ksplit == 1 && epilogue == EPI_SWIGLU) return p;
        p.nb = (mt == 1 && KB > 256) ? 2 : 4;   // with several row strips the activation re-reads dominate: 4 strips
        if (max_ksplit == 1 && mt == 1) p.nb = 2;
        const int groups = (N / 16 + p.nb - 1) / p.nb;
        while (groups * p.ksplit < 512 && p.ksplit * 2 <= max_ksplit && p.ksplit < kSmallMaxKsplit &&
               KB / (p.ksplit * 2 * 4) >= 4)
            p.ksplit *= 2;
        return p;
    }
    // Tiled kernel.  Many tiles (prompt forwards): 4-wave workgroups, two per CU, no slicing.  Few tiles
    // (short prompt forwards; decode batches of 65-256 rows on matrices too small for the sweep kernel): measured on the 7B shapes, outer k-slices up to 4 (partial sums
    // through HBM are small while rows are few) beat everything else; where slicing is impossible an
    // 8-wave workgroup halves the k range inside the workgroup instead.
    // Tile height: 64 token-rows, or 128 from kTiledTallFrom rows on.  A 64 x 256 tile asks L2 for 20 KiB per 16
    // matrix-core instructions of every wave, which is more than a compute unit can take in while its matrix cores
    // run; a 128 x 256 tile asks for 24 KiB per 32.  Below that row count tall tiles leave too many rows idle.
    p.tms = (m_rows >= kTiledTallFrom && g_tall_tiles.load(std::memory_order_relaxed)) ? 8 : 4;
    const int tiles = ((N + 255) / 256) * ((m_rows + p.tms * 16 - 1) / (p.tms * 16));
    // Measured at the 7B shape, same GPU, against slicing up to 512 workgroups whenever there are fewer than 512 tiles:
    // prompt forward of 640 token-rows 12.6 against 13.8 ms (q|k|v, 480 tiles, now unsliced; o and down, 160 tiles, two
    // slices instead of four), 1280 token-rows 19.6 against 21.9, decode steps of 129-256 rows (run by this kernel at the time) 3-4 % shorter; stopping at
    // 256 workgroups instead of 320 costs 4 % at 1024 token-rows, going on to 384 costs 5 % at 640 and 1280.
    if (tiles >= kTiledNoSliceTiles) return p;
    while (tiles * p.ksplit < kTiledFullGroups && p.ksplit * 2 <= max_ksplit && p.ksplit < kTiledMaxKsplit &&
           KB / (p.ksplit * 2) >= 16)
        p.ksplit *= 2;
    if (p.ksplit == 1) p.kp = 2;
    return p;
}

size_t gemm_partial_rows_bound(int N, int n_max, bool sliced_only)
{
    // up to kSweepMaxRows rows: at most kSmallMaxKsplit slices; above: the tiled kernel slices only while it
    // has fewer than kTiledNoSliceTiles tiles, i.e. up to 128 * floor((kTiledNoSliceTiles - 1) / column tiles) rows
    // (its tallest tile)
    const size_t n = (size_t)std::max(n_max, 1);
    const size_t col_tiles = (size_t)(N + 255) / 256;
    const size_t tiled_rows = 128 * ((size_t)(kTiledNoSliceTiles - 1) / std::max<size_t>(col_tiles, 1));
    size_t need = sliced_only ? 1 : n;
    need = std::max(need, (size_t)kSmallMaxKsplit * std::min<size_t>(n, (size_t)kSweepMaxRows));
    need = std::max(need, (size_t)kTiledMaxKsplit * std::min(n, tiled_rows));
    return need;
}

}  // namespace ss
