// Internal host-side declarations shared by the API translation unit and the kernel
// translation units.  Nothing here is visible at the C boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "igemm.hpp"

namespace unit {

// Tile shapes compiled into the library.  Each exists for int8 and fp16, with and
// without the conv gather.
struct TileCfg {
    int bm, bn, bkb;          // workgroup tile rows / cols / reduction bytes per step
    int wgm, wgn, wgk;        // wave grid
    int mf;                   // MFMA edge
    int nst;                  // LDS stages
};
enum { NUM_TILES = 13 };
extern const TileCfg g_tiles[NUM_TILES];
extern const TileCfg g_tiles_fp8[NUM_TILES];   // same tiles, wave grids of the fp8 kernels

struct TileChoice {
    int tile;                 // index into g_tiles
    int split_k;              // grid.z
    int ksteps_per_split;
    int workgroups;
};

// selector.cpp (pure host arithmetic)
// bsrc: where the B operand comes from (BSRC_*); the tile depends on the shape only, the split also on bsrc
// cb: 16-byte channel chunks per pixel (BSRC_NCHWS only: its steps must divide them), 0 = not applicable
TileChoice select_tile(int rows, int cols, int kchunks, int dtype, int bsrc, bool allow_split = true, int cb = 0);
// A problem as one or two column ranges, each with a tile shape of its own.  Large problems whose count of
// 256 x 256 tiles leaves the last round of workgroups partly empty get their whole rounds as one launch and
// the remaining columns as a second launch with a narrower tile that fits them into one round.
struct RangePlan {
    int n;                    // 1 or 2 launches
    int col_begin[2], col_end[2];
    TileChoice choice[2];
};
RangePlan plan_ranges(int rows, int cols, int kchunks, int dtype, int bsrc, bool allow_split, int cb, bool allow_ranges);
// test / sweep hook behind unit_debug_force_tile: tile and grid split every later select_tile returns (-1 = the rule)
void force_tile(int tile, int split);
bool tile_is_forced();
// whether `tile` has a kernel for this public dtype and B source (LDS footprint, vmcnt range)
bool tile_fits(int tile, int dtype, int bsrc);

// launchers (kernels_*.hip).  All return hipError_t from the launch.
hipError_t launch_igemm(int dtype, int bsrc, int tile, const IgemmArgs &a, int split_k, hipStream_t st);

hipError_t launch_pack_act(int dtype, int n, int c, int h, int w, const void *x, void *xp, hipStream_t st);
hipError_t launch_pack_act_sub(int dtype, int n, int c, int h, int w, int sh, int sw, int p, int q,
                               const void *x, void *xp, hipStream_t st);
hipError_t launch_pack_weights(int dtype, int k, int c, int r, int s, const void *w, void *wp, hipStream_t st);
hipError_t launch_unpack_act_i8(int n, int c, int h, int w, const void *xp, int8_t *x, hipStream_t st);
hipError_t launch_pad_rows(const void *src, long ld_bytes, int rows, int row_bytes,
                           void *dst, int dst_row_bytes, hipStream_t st);

// out[r] = 128 * sum of the signed bytes of row r (rows 16-byte aligned, chunks*16 bytes long)
hipError_t launch_rowsum128_i8(const void *m, long ld, int rows, int chunks, int32_t *out, hipStream_t st);

// register-resident MFMA loop (measurement aid); out: 256 * 8 waves * 4 counters of 8 bytes
hipError_t launch_mfma_ceiling(int dtype, int steps, int random_operands, void *out, hipStream_t st);

// matmul with at most UNIT_GEMV_MAX_ROWS rows on the vector ALU's dot-product instructions (DT_I8 / DT_F16)
enum { GEMV_MAX_ROWS = 4 };      // (measured: from 8 rows on the 16 x 64 MFMA tile is as fast or faster)
hipError_t launch_gemv(int dtype, const void *A, long lda, const void *B, long ldb, int m, int n, int kchunks,
                       void *C, long ldc, hipStream_t st);

struct ReduceArgs {
    const void *partials;  int nsplit;  long split_stride;      // elements
    int dtype;
    long total;                                                  // n*k*pq output elements
    int K, PQ;                                                   // channel = (idx / PQ) % K
    void *out;                                                   // int32 / float or NULL
    int epi;  const float *scale;  const int32_t *bias;  const int32_t *residual;  int relu;
    const int8_t *res_packed;  int res_mult;                     // [n*pq][packed_ld] int8 residual, or NULL
    int8_t *out_i8;  int8_t *out_packed;  int packed_ld;
};
hipError_t launch_splitk_reduce(const ReduceArgs &a, hipStream_t st);

hipError_t launch_maxpool_packed_i8(int n, int cp, int h, int w, int window, int stride, int pad,
                                    int p, int q, const void *x, void *y, hipStream_t st);
hipError_t launch_avgpool_packed_i8(int n, int c, int cp, int hw, const void *x, const float *scale,
                                    int8_t *y, hipStream_t st);
hipError_t launch_widen_residual_i8(int n, int c, int cp, int hw, const void *x, int mult,
                                    int32_t *res, hipStream_t st);

}  // namespace unit
