// Implicit-GEMM main kernel for gfx950 MFMA: D[row][col] = sum_k A[row][k] * B[col][k].
//
// Both operands are "rows of reduction-contiguous bytes".  For conv2d the A operand is
// the packed weight matrix (row = output channel) and the B operand is gathered on the
// fly from the packed NHWC activations (col = output pixel, never materialised im2col);
// for matmul both are plain matrices.  Rows land on MFMA rows and columns on MFMA
// columns, so adjacent lanes hold adjacent pixels / matmul n and NCHW / row-major stores
// are contiguous per lane group.
//
// This is the hand-made counterpart of what the paper's Rewriter does (Section III-C):
// the reduction loops are tiled by the instruction's trip counts and made innermost, the
// "operand generation" step becomes the global -> LDS -> VGPR fragment path, the p x p
// accumulator window (Section III-C.3, GPU tuning) becomes the TM x TN grid of MFMA
// accumulators per wave, H and W are always fused into one pixel index, and the
// reduction can be split across waves of a workgroup and across workgroups.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace unit {

typedef int      v4i  __attribute__((ext_vector_type(4)));
typedef int      v16i __attribute__((ext_vector_type(16)));
typedef float    v4f  __attribute__((ext_vector_type(4)));
typedef float    v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h  __attribute__((ext_vector_type(8)));

enum { DT_I8 = 0, DT_F16 = 1 };
enum { EPI_RAW = 0, EPI_REQUANT = 1 };

struct IgemmArgs {
    // operands (byte pointers; every row starts 16-byte aligned, reduction zero padded to 16 B)
    const uint8_t *A;  long lda;  int rows;        // lda in bytes
    const uint8_t *B;  long ldb;  int cols;        // plain B: ldb in bytes
    int kchunks;                                    // reduction length in 16-byte chunks
    int ksteps_per_split;                           // main-loop steps per grid.z slice
    // conv gather of B (CONV kernels only): packed activations [n][H][W][CB*16 bytes]
    int H, W, CB, P, Q, PQ, R, S, sh, sw, ph, pw;
    // output: element (row, col) of image n = col / cols_per_img lives at
    //   out[n*img_stride + row*row_stride + col % cols_per_img]   (4-byte elements)
    void *out;  long row_stride;  long img_stride;  int cols_per_img;
    long split_stride;                              // elements between grid.z partials
    long b_bytes;                                   // conv: bytes of the packed activation tensor (< 2 GiB)
    // fused epilogue (EPI_REQUANT): int8 results
    int epi;
    const float *scale;  const int32_t *bias;  const int32_t *residual;  int relu;
    int8_t *out_i8;                                 // same indexing as out, or NULL
    int8_t *out_packed;  int packed_ld;             // [col][packed_ld] int8, or NULL
    int store_raw;                                  // also store raw accumulators to out
};

// One element of the requantise rule.  v_cvt_f32_i32 and v_rndne_f32 both round to
// nearest even; the multiply is a single fp32 operation (no fused add exists here).
__device__ __forceinline__ int requant_elem(int t, float scale, int relu)
{
    float g = __fmul_rn((float)t, scale);
    float i = rintf(g);
    if (relu) i = fmaxf(i, 0.0f);
    i = fminf(fmaxf(i, -128.0f), 127.0f);
    return (int)i;
}

template <int DT, int MF> struct Mma;
template <> struct Mma<DT_I8, 32> {
    typedef v16i acc_t;  typedef int elem_t;  enum { NACC = 16 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }
};
template <> struct Mma<DT_I8, 16> {
    typedef v4i acc_t;  typedef int elem_t;  enum { NACC = 4 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0); }
};
template <> struct Mma<DT_F16, 32> {
    typedef v16f acc_t;  typedef float elem_t;  enum { NACC = 16 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0); }
};
template <> struct Mma<DT_F16, 16> {
    typedef v4f acc_t;  typedef float elem_t;  enum { NACC = 4 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0); }
};

// Row of accumulator element e held by `lane` inside one MFMA tile (column is lane % MF).
template <int MF> __device__ __forceinline__ int acc_row(int e, int lane)
{
    if (MF == 32) return 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
    return 4 * (lane >> 4) + e;
}

// LDS tile layout: row-major rows of BKB bytes, 16-byte chunks XOR-swizzled by row so
// that the 16 lanes served together by a 128-bit LDS access always touch 16 different
// 16-byte bank groups (256 bytes = all 64 banks).
template <int NCH> __device__ __forceinline__ int swz(int row)
{
    constexpr int SWD = (NCH >= 16) ? 1 : 16 / NCH;
    return (row / SWD) % NCH;
}

// Raw buffer descriptors: loads and stores that fall outside [0, num_records) return zero /
// are dropped by the hardware, so tile edges, the reduction tail and conv padding need no
// branches -- an invalid lane just gets an offset beyond the range.
typedef unsigned v4u __attribute__((ext_vector_type(4)));
#define UNIT_OOB 0x80000000u      /* every buffer is kept below 2 GiB by the host checks */

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ unsigned to_bits(int v)   { return (unsigned)v; }
__device__ __forceinline__ unsigned to_bits(float v) { return __float_as_uint(v); }
__device__ __forceinline__ v4i buf_load16(__amdgpu_buffer_rsrc_t r, unsigned off)
{
    return __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0));
}

template <int DT, int BM, int BN, int BKB, int WGM, int WGN, int WGK, int MF, bool CONV>
struct IgemmCfg {
    enum {
        NT    = WGM * WGN * WGK * 64,
        NCH   = BKB / 16,
        WTM   = BM / WGM,  WTN = BN / WGN,
        TM    = WTM / MF,  TN  = WTN / MF,
        KSUBB = (MF == 32) ? 32 : 64,              // reduction bytes per MFMA
        NKSUB = BKB / KSUBB,
        CPL   = KSUBB / 16,                        // 16-byte chunks per MFMA along k
        LA    = (BM * NCH + NT - 1) / NT,
        LB    = (BN * NCH + NT - 1) / NT,
        STAGE_BYTES  = (BM + BN) * BKB,
        REDUCE_BYTES = (WGK - 1) * BM * BN * 4,
        SMEM_BYTES   = (2 * STAGE_BYTES > REDUCE_BYTES) ? 2 * STAGE_BYTES : REDUCE_BYTES,
    };
    static_assert(BM % (WGM * MF) == 0 && BN % (WGN * MF) == 0, "wave tiles must be whole MFMA tiles");
    static_assert(NKSUB % WGK == 0 && NKSUB >= WGK, "in-group split must divide the sub-steps");
    static_assert(BKB % KSUBB == 0, "step must be whole MFMAs");
};

template <int DT, int BM, int BN, int BKB, int WGM, int WGN, int WGK, int MF, bool CONV, int EPI>
__global__ void __launch_bounds__(WGM * WGN * WGK * 64)
igemm_kernel(const IgemmArgs g)
{
    typedef IgemmCfg<DT, BM, BN, BKB, WGM, WGN, WGK, MF, CONV> C;
    typedef Mma<DT, MF> M;
    typedef typename M::acc_t acc_t;
    typedef typename M::elem_t elem_t;
    constexpr int NT = C::NT, NCH = C::NCH, TM = C::TM, TN = C::TN, LA = C::LA, LB = C::LB;
    constexpr bool FULL_A = (BM * NCH) % NT == 0, FULL_B = (BN * NCH) % NT == 0;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wk   = wave / (WGM * WGN);
    const int wm   = (wave % (WGM * WGN)) / WGN;
    const int wn   = wave % WGN;

    // ---- tile coordinates.  Workgroups are dealt round-robin to the 8 XCDs (each with
    // its own L2): give every XCD one contiguous run of the tile order, and walk that
    // order in bands of 8 row-tiles so the tiles resident together share A and B rows.
    const int tiles_m = (g.rows + BM - 1) / BM;
    const int tiles_n = (g.cols + BN - 1) / BN;
    const int ntiles  = tiles_m * tiles_n;
    int bid = blockIdx.x;
    if ((ntiles & 7) == 0) bid = (bid & 7) * (ntiles >> 3) + (bid >> 3);
    constexpr int BAND = 8;
    const int band      = bid / (BAND * tiles_n);
    const int band_m0   = band * BAND;
    const int band_rows = (tiles_m - band_m0 < BAND) ? tiles_m - band_m0 : BAND;
    const int in_band   = bid - band * BAND * tiles_n;
    const int tm = band_m0 + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int row0 = tm * BM, col0 = tn * BN;

    const int ksteps_total = (g.kchunks + NCH - 1) / NCH;
    const int ks_begin = blockIdx.z * g.ksteps_per_split;
    int ks_end = ks_begin + g.ksteps_per_split;
    if (ks_end > ksteps_total) ks_end = ksteps_total;

    // ---- per-thread global-load bookkeeping: chunk slot id = tid + i*NT -> (row r, chunk cB).
    // NT is a multiple of NCH, so every slot of a thread has the same chunk column cB.
    const int cB = tid % NCH;
    const int rows_here = (g.rows - row0 < BM) ? g.rows - row0 : BM;
    const __amdgpu_buffer_rsrc_t rsA =
        make_rsrc(g.A + (long)row0 * g.lda, (unsigned)((long)(rows_here - 1) * g.lda + (long)g.kchunks * 16));
    unsigned offA[LA];  int ldsA[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int id = tid + i * NT;
        int r = id / NCH;
        bool in_tile = FULL_A || (id < BM * NCH);
        offA[i] = (in_tile && r < rows_here) ? (unsigned)(r * (int)g.lda + cB * 16) : UNIT_OOB;
        ldsA[i] = in_tile ? r * BKB + ((cB ^ swz<NCH>(r)) << 4) : -1;
    }
    const int cols_here = (g.cols - col0 < BN) ? g.cols - col0 : BN;
    const __amdgpu_buffer_rsrc_t rsB = CONV
        ? make_rsrc(g.B, (unsigned)g.b_bytes)
        : make_rsrc(g.B + (long)col0 * g.ldb, (unsigned)((long)(cols_here - 1) * g.ldb + (long)g.kchunks * 16));
    unsigned offB[LB];  int ldsB[LB];
    int bh0[LB], bw0[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        int id = tid + i * NT;
        int r = id / NCH;
        bool in_tile = FULL_B || (id < BN * NCH);
        bool valid = in_tile && r < cols_here;
        ldsB[i] = in_tile ? BM * BKB + r * BKB + ((cB ^ swz<NCH>(r)) << 4) : -1;
        if (CONV) {
            int cc = valid ? col0 + r : 0;
            int n = cc / g.PQ, pq = cc - n * g.PQ;
            int p = pq / g.Q, q = pq - p * g.Q;
            // an invalid column gets a row far outside the image: its bounds test always fails
            const int bh = p * g.sh - g.ph, bw = q * g.sw - g.pw;
            bh0[i] = valid ? bh : -0x100000;
            bw0[i] = bw;
            // byte offset of tap (0,0); modulo 2^32 (negative in the padding), exact once a tap is in range
            offB[i] = (unsigned)((n * g.H + bh) * g.W + bw) * (unsigned)(g.CB * 16);
        } else {
            offB[i] = valid ? (unsigned)(r * (int)g.ldb + cB * 16) : UNIT_OOB;
            bh0[i] = bw0[i] = 0;
        }
    }
    // conv: reduction chunk kc -> (r, s, channel chunk cb), advanced incrementally per step
    int kc = ks_begin * NCH + cB;
    int cr = 0, cs = 0, ccb = 0;
    if (CONV) {
        int rs = kc / g.CB;
        ccb = kc - rs * g.CB;
        cr = rs / g.S;
        cs = rs - cr * g.S;
    }

    v4i ra[LA], rb[LB];

    // loads the tile of the step whose first chunk (for this thread) is kc, then advances kc
    auto load_global = [&]() {
        const bool kok = kc < g.kchunks;
        const unsigned kbyte = (unsigned)(kc - cB) * 16u;          // = step * BKB
#pragma unroll
        for (int i = 0; i < LA; ++i)
            ra[i] = buf_load16(rsA, kok ? offA[i] + kbyte : UNIT_OOB);
        if (CONV) {
            const unsigned tap = (unsigned)((cr * g.W + cs) * g.CB + ccb) * 16u;
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                int h = bh0[i] + cr, w = bw0[i] + cs;
                bool ok = kok && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
                rb[i] = buf_load16(rsB, ok ? offB[i] + tap : UNIT_OOB);
            }
            ccb += NCH;
            while (ccb >= g.CB) {
                ccb -= g.CB;
                if (++cs == g.S) { cs = 0; ++cr; }
            }
        } else {
#pragma unroll
            for (int i = 0; i < LB; ++i)
                rb[i] = buf_load16(rsB, kok ? offB[i] + kbyte : UNIT_OOB);
        }
        kc += NCH;
    };
    auto store_lds = [&](int buf) {
        uint8_t *base = smem + buf * C::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < LA; ++i)
            if (FULL_A || ldsA[i] >= 0) *reinterpret_cast<v4i *>(base + ldsA[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i)
            if (FULL_B || ldsB[i] >= 0) *reinterpret_cast<v4i *>(base + ldsB[i]) = rb[i];
    };

    // ---- fragment addressing (lane -> row inside an MFMA tile, 16-byte chunk along k)
    const int lrow   = lane % MF;
    const int lchunk = lane / MF;                   // 0..CPL-1
    const int a_row  = wm * C::WTM + lrow;
    const int b_row  = wn * C::WTN + lrow;
    const int a_swz  = swz<NCH>(a_row);             // unchanged by +MF*i (multiples of 16)
    const int b_swz  = swz<NCH>(b_row);

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < M::NACC; ++e) acc[i][j][e] = 0;

    if (ks_begin < ks_end) {
        load_global();
        store_lds(0);
        __syncthreads();
        for (int ks = ks_begin; ks < ks_end; ++ks) {
            const int buf = (ks - ks_begin) & 1;
            const bool more = ks + 1 < ks_end;
            if (more) load_global();
            const uint8_t *sA = smem + buf * C::STAGE_BYTES;
            const uint8_t *sB = sA + BM * BKB;
#pragma unroll
            for (int kk = 0; kk < C::NKSUB / WGK; ++kk) {
                const int ksub = kk * WGK + wk;
                const int ch = ksub * C::CPL + lchunk;
                v4i af[TM], bf[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    af[i] = *reinterpret_cast<const v4i *>(sA + (a_row + i * MF) * BKB + ((ch ^ a_swz) << 4));
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    bf[j] = *reinterpret_cast<const v4i *>(sB + (b_row + j * MF) * BKB + ((ch ^ b_swz) << 4));
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        M::run(acc[i][j], af[i], bf[j]);
            }
            if (more) store_lds(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- in-group split reduction: waves with wk > 0 park their accumulators in LDS
    // (lane-contiguous, conflict free), wave slice 0 adds them in fixed order.
    if (WGK > 1) {
        elem_t *red = reinterpret_cast<elem_t *>(smem);
        const int wmn = wave % (WGM * WGN);
        if (wk > 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < M::NACC; ++e)
                        red[((((wk - 1) * WGM * WGN + wmn) * TM * TN + i * TN + j) * M::NACC + e) * 64 + lane] = acc[i][j][e];
        }
        __syncthreads();
        if (wk > 0) return;
        for (int k2 = 1; k2 < WGK; ++k2)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < M::NACC; ++e)
                        acc[i][j][e] += red[((((k2 - 1) * WGM * WGN + wmn) * TM * TN + i * TN + j) * M::NACC + e) * 64 + lane];
    }

    // ---- epilogue
    if (EPI == EPI_RAW) {
        // 4-byte stores through a buffer descriptor anchored at the tile's first row;
        // out-of-tile lanes get an out-of-range offset and are dropped by the hardware.
        const elem_t *tile_base = reinterpret_cast<const elem_t *>(g.out) + (long)blockIdx.z * g.split_stride +
                                  (long)row0 * g.row_stride;
        const __amdgpu_buffer_rsrc_t rsO = make_rsrc(tile_base, UNIT_OOB);   // lanes are masked explicitly
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col0 + wn * C::WTN + j * MF + lrow;
            unsigned cbase;
            if (CONV) {
                int n = col / g.cols_per_img;
                cbase = (unsigned)((long)n * g.img_stride + (col - n * g.cols_per_img));
            } else {
                cbase = (unsigned)col;
            }
            const bool col_ok = col < g.cols;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int e = 0; e < M::NACC; ++e) {
                    const int lr = wm * C::WTM + i * MF + acc_row<MF>(e, lane);
                    const bool ok = col_ok && lr < rows_here;
                    const unsigned off = ok ? (cbase + (unsigned)lr * (unsigned)g.row_stride) * 4u : UNIT_OOB;
                    const elem_t val = acc[i][j][e];
                    __builtin_amdgcn_raw_buffer_store_b32(to_bits(val), rsO, off, 0, 0);
                }
            }
        }
    } else {
        elem_t *out = reinterpret_cast<elem_t *>(g.out);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col0 + wn * C::WTN + j * MF + lrow;
            if (col >= g.cols) continue;
            long cbase;
            if (CONV) {
                int n = col / g.cols_per_img;
                cbase = (long)n * g.img_stride + (col - n * g.cols_per_img);
            } else {
                cbase = col;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int e = 0; e < M::NACC; ++e) {
                    const int row = row0 + wm * C::WTM + i * MF + acc_row<MF>(e, lane);
                    if (row >= g.rows) {
                        // padding channels of a packed int8 output are defined to be zero
                        if (g.out_packed && row < g.packed_ld) g.out_packed[(long)col * g.packed_ld + row] = 0;
                        continue;
                    }
                    const long addr = cbase + (long)row * g.row_stride;
                    int t = (int)acc[i][j][e];
                    if (g.store_raw) out[addr] = acc[i][j][e];
                    if (g.bias) t += g.bias[row];
                    if (g.residual) t += g.residual[addr];
                    int v = requant_elem(t, g.scale[row], g.relu);
                    if (g.out_i8) g.out_i8[addr] = (int8_t)v;
                    if (g.out_packed) g.out_packed[(long)col * g.packed_ld + row] = (int8_t)v;
                }
            }
        }
    }
}

}  // namespace unit
