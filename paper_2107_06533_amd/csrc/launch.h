// Host-callable launchers of the gfx950 kernels (implemented in the .hip files).
#pragma once
#include "common.h"

namespace kfac {

void launch_tile_any(const TileDesc* descs, const TileJob* jobs, int njobs, int xcd_order, hipStream_t s);
void launch_tile_gemm(const TileDesc* descs, const TileJob* jobs, int njobs, int xcd_order, hipStream_t s);
void launch_tile_gemm_pad(const TileDesc* descs, const TileJob* jobs, int njobs, int pad_bytes, hipStream_t s);
// row-major x row-major products only (both operands OP_KMAJOR without ones column): direct-to-LDS loop
void launch_tile_gemm_dl(const TileDesc* descs, const TileJob* jobs, int njobs, hipStream_t s);
// row-major x row-major products that give way to latency-critical workgroups on their compute unit (cu_flags may be null)
// deep: 32-deep panels (64 KB of LDS) for launches that run one workgroup to a compute unit, else 16-deep (32 KB)
int deep_lds_extra();   // bytes of LDS the deep variant uses beyond the other
void launch_tile_gemm_yield(const TileDesc* descs, const TileJob* jobs, int njobs, int pad_bytes, const int* cu_flags, bool deep, hipStream_t s);
// the same on jobs that each cover one 32-column block of a tile (TileJob::quarter = 1 + block); direct jobs only
void launch_tile_gemm_quarter(const TileDesc* descs, const TileJob* jobs, int njobs, int* cu_flags, hipStream_t s);
void launch_tile_reduce(const TileDesc* descs, const ReduceJob* jobs, int njobs, hipStream_t s);
// pair_jobs: tiles of lag_pair_rows() x lag_pair_cols() channel pairs (bi, bj) that hold a pair c2 <= c, the
// bias pseudo-channel C included; mirror_jobs: 64 x 64 tiles bi >= bj of the factor
void launch_lag_assemble(const LagAsm* lags, const LagJob* pair_jobs, int npair, const LagJob* mirror_jobs, int nmirror, hipStream_t s);
int lag_pair_rows();
int lag_pair_cols();

void launch_gj_init(const InvMat* mats, const void* jobs, int njobs, float gamma, hipStream_t s);
// cu_flags (may be null): table of CU_SLOTS words in which the latency-critical workgroups of these
// kernels count themselves while they run, and which their product workgroups give way to
void launch_gj_pivot(const InvMat* mats, const void* jobs, int mat0, int nmats, int step, float gamma, int small, hipStream_t s, int lds_pad = 0,
                     int* cu_flags = nullptr);
void launch_gj_pivot_update(const InvMat* mats, const void* pjobs, int npiv, int step, float gamma,
                            const TileDesc* descs, const TileJob* ujobs, int nupd, hipStream_t s, int lds_pad = 0, int* cu_flags = nullptr,
                            int critical = 0);   // critical: the pivot workgroups count themselves in (the update tiles always give way)
void launch_gj_panel(const InvMat* mats, const void* jobs, int njobs, int step, hipStream_t s, int lds_pad = 0, int* cu_flags = nullptr);
int cu_flag_slots();
void launch_gj_qmirror(const InvMat* mats, const void* jobs, int njobs, hipStream_t s);
void launch_gj_move(const PanelMove* moves, const void* jobs, int njobs, int kchunks, int to_matrix, hipStream_t s);
void launch_tri_pack(const PackMat* mats, const void* jobs, int njobs, float* packed, int to_full, hipStream_t s);
void launch_gj_finish(const InvMat* mats, const void* jobs, int njobs, hipStream_t s);

}  // namespace kfac
