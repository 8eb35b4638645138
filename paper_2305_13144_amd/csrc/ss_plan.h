// Launch planning of the projection kernels: plain host arithmetic, no HIP types, so that it can be
// compiled and checked on a machine without a GPU.
#ifndef SS_PLAN_H
#define SS_PLAN_H

#include <cstddef>

namespace ss {

enum Epilogue { EPI_PARTIAL = 0, EPI_SWIGLU = 1 };

constexpr int kSweepMaxRows = 256;   // 16 row strips: accumulators and the LDS chunk of the sweep kernel still fit

struct GemmPlan {
    int ksplit, nb, kd, kp;
    int sweep_p, sweep_gn;
    int sweep_kh;   // sweep kernel: waves per unit (1 or 2)
    int tms;        // tiled kernel: row strips per tile (4 = 64 rows, 8 = 128 rows)
};

constexpr int kTiledTallFrom = 896;   // token-rows from which the tiled kernel uses 128-row tiles

// n_cu: compute units of the device (the sweep kernel runs one workgroup per unit).
// max_ksplit: 1 when the consumer reads the output directly (logits).
GemmPlan gemm_plan(int N, int Kp, int m_rows, int epilogue, int n_cu, int max_ksplit = 8);

// Strips per wave of the sweep kernel for this epilogue and row count.
int sweep_nbw(int epilogue, int m_rows);

// Rows a [ksplit][rows][N] partial-sum buffer must hold so that every plan gemm_plan can return for an
// [N, *] matrix and 1 <= m_rows <= n_max fits: an upper bound of ksplit * m_rows over that range.
// sliced_only: count only plans with ksplit > 1 (a buffer that is used only then).
size_t gemm_partial_rows_bound(int N, int n_max, bool sliced_only = false);

// Testing aid: 0 = choose per shape (default), 1 = never use the sweep kernel, 2 = use it for every
// projection of at most kSweepMaxRows rows.
void set_gemm_mode(int mode);
int gemm_mode();

}  // namespace ss

#endif
