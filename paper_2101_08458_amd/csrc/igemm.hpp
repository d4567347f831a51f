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
typedef int      v2i  __attribute__((ext_vector_type(2)));
typedef short    v4s  __attribute__((ext_vector_type(4)));
typedef int      v8i  __attribute__((ext_vector_type(8)));
typedef int      v16i __attribute__((ext_vector_type(16)));
typedef float    v4f  __attribute__((ext_vector_type(4)));
typedef float    v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h  __attribute__((ext_vector_type(8)));
typedef __bf16   v8bf __attribute__((ext_vector_type(8)));

// Operand types.  The matrix unit multiplies signed bytes only; an unsigned-byte operand u is
// fed as u - 128 (its bytes XORed with 0x80 on the way into the fragments) and the caller
// supplies 128 * (sum of the other operand along the reduction) as an additive correction:
// DT_U8A has the unsigned operand on the A side (correction per output column), DT_U8B on
// the B side (correction per output row).  Bytes the hardware zero-fills (reduction tail,
// conv padding) become -128 the same way; the other operand is zero on the tail, and for
// conv padding the correction sums every tap, so both cancel exactly.
// DT_FP8 (OCP E4M3) uses the 32-byte-per-lane MFMAs: its fragments are two 16-byte chunks wide.
enum { DT_I8 = 0, DT_F16 = 1, DT_BF16 = 2, DT_U8A = 3, DT_U8B = 4, DT_FP8 = 5 };
enum { EPI_RAW = 0, EPI_REQUANT = 1 };
// where the B operand (columns) comes from: a plain matrix, the packed-NHWC conv gather, or
// an NCHW tensor read directly (1x1 stride-1 unpadded convs: channel rows of pixels,
// transposed on the way from LDS into the fragments).  BSRC_NCHWS is the general form of the
// direct read for stride 1 with "same" padding: output pixel m of the flattened
// image needs input pixel m + delta(tap) of every channel, so the B tile of a step is a window of
// each channel row shifted by the tap's delta.  The 16-byte loads start at the window's exact byte (any
// offset), so the tile lands in LDS as in the 1x1 mode and is read the same way; pixels whose tap
// falls into the padding are masked after the read, and the two chunks that straddle the tensor's
// start and end are patched from a copy of its first and last 16 bytes.
// BSRC_GATHERU is the gather for layers whose pixels hold a whole number of steps of channel chunks: every lane
// of a step then works on the same tap and the tap walk is scalar (the launcher picks it; callers say BSRC_GATHER).
// BSRC_NCHWE is the 1x1 direct read for rows that are not dword-aligned (IgemmArgs::edge; picked by the launcher).
enum { BSRC_PLAIN = 0, BSRC_GATHER = 1, BSRC_NCHW = 2, BSRC_NCHWS = 3, BSRC_GATHERU = 4, BSRC_NCHWE = 5 };

// Divisor with its reciprocal for the kernels' integer divisions: m = floor(2^32 / d) (0xffffffff for d = 1).
// The host fills these in; a division is then a multiply-high and one correction (see divu).
struct DivU { unsigned d, m; };

struct IgemmArgs {
    // operands (byte pointers; every row starts 16-byte aligned, reduction zero padded to 16 B)
    const uint8_t *A;  long lda;  int rows;        // lda in bytes
    const uint8_t *B;  long ldb;  int cols;        // plain B: ldb in bytes
    int kchunks;                                    // reduction length in 16-byte chunks
    int ksteps_per_split;                           // main-loop steps per grid.z slice
    // conv gather of B (CONV kernels only): packed activations [n][H][W][CB*16 bytes]
    // (D, T, sd, pd describe the depth axis; conv2d is D = T = 1)
    int D, H, W, CB, P, Q, PQ, T, R, S, sd, sh, sw, pd, ph, pw;
    int Cin;                                        // NCHW-direct kernels: real channel count
    int row_runs;                                   // tile order: consecutive workgroups of an XCD share a row tile
    int edge;                                       // NCHW-direct 1x1: rows are not dword-aligned, so the 16-byte chunk
                                                    // that crosses the tensor's end is not loaded but patched (see read_frags)
    int per_img;                                    // NCHW-direct: column tiles never straddle images (each image's
                                                    // pixels are tiled on their own; needed when an image does not
                                                    // hold a whole number of 16-byte pixel chunks)
    // output: element (row, col) of image n = col / cols_per_img lives at
    //   out[n*img_stride + row*row_stride + col % cols_per_img]   (4-byte elements)
    void *out;  long row_stride;  long img_stride;  int cols_per_img;
    long split_stride;                              // elements between grid.z partials
    long b_bytes;                                   // conv: bytes of the packed activation tensor (< 2 GiB)
    // fused epilogue (EPI_REQUANT): int8 results
    int epi;
    const float *scale;  const int32_t *bias;  const int32_t *residual;  int relu;
    const int8_t *res_packed;  int res_mult;        // int8 residual [col][packed_ld] times res_mult, or NULL
    int8_t *out_i8;                                 // same indexing as out, or NULL
    int8_t *out_packed;  int packed_ld;             // [col][packed_ld] int8, or NULL
    int store_raw;                                  // also store raw accumulators to out
    // divisors of the index arithmetic (unused ones hold d = 1)
    DivU dv_pq, dv_ppq, dv_q, dv_w;                 // PQ (output pixels per image), P*Q, Q, W
    DivU dv_cpi;                                    // cols_per_img
    DivU dv_tiles_n, dv_band, dv_tiles_img;         // column tiles, 8 * column tiles, column tiles per image (per_img)
    int nimg;                                       // cols / PQ (images)
    // (appended: the order of the fields above decides how the compiler groups the argument loads of every kernel's
    // prologue; inserting these three in front of dv_tiles_n, or sorting all fields by use into 64-byte lines, cost
    // 3-4 % of the batch-1 step each time it was tried)
    DivU dv_cb, dv_s, dv_r;                         // CB, S, R (the per-lane tap walk of the gather)
    // column range this launch tiles: [col_base, col_limit) of the cols columns (one launch: 0 and cols; a problem
    // whose tile count leaves the last round of workgroups mostly empty is launched as two ranges with two tile shapes)
    int col_base, col_limit;
#ifdef UNIT_PROBE
    // instrumented build only (make probe): per wave 16 x 8 bytes of time stamps, see UNIT_STAMP
    unsigned long long *probe;
#endif
};

// Instrumented build (make probe -> libunit_probe.so, never the product library): every wave stamps the core cycle
// counter and the 100 MHz real-time counter at the kernel's phase boundaries -- 0 entry, 6 prologue arithmetic done,
// 7 first tiles requested, 1 first tile landed (loop start), 2 loop end, 3 ring drained, 4 epilogue stores issued,
// 5 stores acknowledged -- and writes them to probe[(workgroup * waves + wave) * 16 + i] (cycles) and [... + 8 + i]
// (real time) at the end.  Compiled out of the product.
#ifdef UNIT_PROBE
#define UNIT_STAMP(i) do { if (g.probe) { unit_pt[i] = __builtin_readcyclecounter(); unit_pr[i] = __builtin_amdgcn_s_memrealtime(); } } while (0)
// (small-tile step loop only) cycles a wave spends waiting for its own loads / at the barrier / for its fragment reads,
// summed over the steps (the cycle counter is a scalar memory read: its result is only used after the fragment wait)
#define UNIT_CYC() ((unsigned)__builtin_readcyclecounter())
#define UNIT_ACC(sum, from, to) do { sum += (to) - (from); } while (0)
#else
#define UNIT_STAMP(i) do { } while (0)
#endif

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
    typedef v16i acc_t;  typedef int elem_t;  typedef v4i frag_t;  enum { NACC = 16, FW = 1 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }
};
template <> struct Mma<DT_I8, 16> {
    typedef v4i acc_t;  typedef int elem_t;  typedef v4i frag_t;  enum { NACC = 4, FW = 1 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0); }
};
template <> struct Mma<DT_F16, 32> {
    typedef v16f acc_t;  typedef float elem_t;  typedef v4i frag_t;  enum { NACC = 16, FW = 1 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0); }
};
template <> struct Mma<DT_F16, 16> {
    typedef v4f acc_t;  typedef float elem_t;  typedef v4i frag_t;  enum { NACC = 4, FW = 1 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0); }
};

template <> struct Mma<DT_BF16, 32> {
    typedef v16f acc_t;  typedef float elem_t;  typedef v4i frag_t;  enum { NACC = 16, FW = 1 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0); }
};
template <> struct Mma<DT_BF16, 16> {
    typedef v4f acc_t;  typedef float elem_t;  typedef v4i frag_t;  enum { NACC = 4, FW = 1 };
    static __device__ __forceinline__ void run(acc_t &c, const v4i &a, const v4i &b)
    { c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0); }
};
// fp8: each lane feeds 32 operand bytes; format selectors 0 = E4M3 for both operands, block
// scales zero = the unscaled form of the instruction
template <> struct Mma<DT_FP8, 32> {
    typedef v16f acc_t;  typedef float elem_t;  typedef v8i frag_t;  enum { NACC = 16, FW = 2 };
    static __device__ __forceinline__ void run(acc_t &c, const v8i &a, const v8i &b)
    { c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0); }
};
template <> struct Mma<DT_FP8, 16> {
    typedef v4f acc_t;  typedef float elem_t;  typedef v8i frag_t;  enum { NACC = 4, FW = 2 };
    static __device__ __forceinline__ void run(acc_t &c, const v8i &a, const v8i &b)
    { c = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0); }
};
template <int MF> struct Mma<DT_U8A, MF> : Mma<DT_I8, MF> {};
template <int MF> struct Mma<DT_U8B, MF> : Mma<DT_I8, MF> {};

// A fragment of FW 16-byte chunks: consecutive logical chunks ch .. ch+FW-1 of one LDS row
// (the swizzle is applied per chunk), or FW*4 assembled words.
// a / b for 0 <= a < 2^22, 0 < b: float reciprocal plus one correction step (a hardware integer
// division is ~40 instructions, and a small kernel's prologue does about ten of them)
__device__ __forceinline__ int div_small(int a, int b)
{
    int q = (int)((float)a * __builtin_amdgcn_rcpf((float)b));
    int r = a - q * b;
    q += (r >= b) ? 1 : 0;
    q -= (r < 0) ? 1 : 0;
    return q;
}
__device__ __forceinline__ int div_any(int a, int b) { return (a < (1 << 22)) ? div_small(a, b) : a / b; }
// n / x.d for any 0 <= n < 2^31: the truncated reciprocal makes the multiply-high at most one too small
__device__ __forceinline__ int divu(int n, DivU x)
{
    const unsigned q = __umulhi((unsigned)n, x.m);
    const unsigned r = (unsigned)n - q * x.d;
    return (int)(q + (r >= x.d ? 1u : 0u));
}

template <int V> struct IntC { static constexpr int value = V; };

template <int FW> struct Frag;
template <> struct Frag<1> {
    static __device__ __forceinline__ v4i load(const uint8_t *row, int ch, int sw)
    { return *reinterpret_cast<const v4i *>(row + ((ch ^ sw) << 4)); }
    static __device__ __forceinline__ v4i pack(const unsigned *w)
    { return v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]}; }
};
template <> struct Frag<2> {
    static __device__ __forceinline__ v8i load(const uint8_t *row, int ch, int sw)
    {
        v4i lo = *reinterpret_cast<const v4i *>(row + ((ch ^ sw) << 4));
        v4i hi = *reinterpret_cast<const v4i *>(row + (((ch + 1) ^ sw) << 4));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    static __device__ __forceinline__ v8i pack(const unsigned *w)
    { return v8i{(int)w[0], (int)w[1], (int)w[2], (int)w[3], (int)w[4], (int)w[5], (int)w[6], (int)w[7]}; }
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

// Global -> LDS without passing through registers: one wave-level instruction moves
// 64 lanes x 16 bytes into 1 KiB of contiguous LDS starting at the (wave-uniform) address
// `lds`; lane L fetches from byte offset `off` of the buffer and lands at lds + 16*L.
// Out-of-range lanes write zeros.  Completion is tracked by vmcnt.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t r, uint8_t *lds, unsigned off)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)lds, 16, off, 0, 0, 0);
}
// Transposing LDS reads (ds_read_b64_tr_b8 / _b16) as inline assembly.  Through the compiler's builtins every such
// read is preceded by s_waitcnt vmcnt(0): the compiler cannot tell which LDS bytes the global -> LDS loads in flight
// will write, so it waits for all of them, which takes the load pipeline down to one tile in flight.  The kernel
// orders tiles and reads itself (stage ring, barriers, explicit vmcnt waits), so it issues these reads unseen by
// that analysis.  The compiler then does not wait for their results either: the kernel waits itself (an s_waitcnt
// the compiler sees, so that its own bookkeeping of the ordinary LDS reads stays exact) and then passes every such
// fragment through lds_tr_done(), an empty statement with the fragment as in/out operand, so that no use of it can
// be scheduled above the wait.
template <int ES, int OFF> __device__ __forceinline__ v2i lds_tr(unsigned lds_addr)
{
    v2i r;
    if (ES == 1) asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(r) : "v"(lds_addr), "n"(OFF) : "memory");
    else         asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(lds_addr), "n"(OFF) : "memory");
    return r;
}
template <typename F> __device__ __forceinline__ void lds_tr_done(F &frag)
{
    asm volatile("" : "+v"(frag));
}
// s_waitcnt lgkmcnt(0) only
#define UNIT_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt((0xF | (0x3 << 14) | (0x7 << 4)))
// s_waitcnt vmcnt(N) lgkmcnt(0)  (expcnt left alone); N <= 63
#define UNIT_WAIT_VM_LGKM0(N) __builtin_amdgcn_s_waitcnt((((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4)))
// s_waitcnt vmcnt(N) only (lgkmcnt and expcnt left alone)
#define UNIT_WAIT_VM(N) __builtin_amdgcn_s_waitcnt((((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8)))
// workgroup barrier that the compiler may not move LDS traffic across
#define UNIT_BARRIER() do { asm volatile("" ::: "memory"); __builtin_amdgcn_s_barrier(); asm volatile("" ::: "memory"); } while (0)

template <int DT, int BM, int BN, int BKB, int WGM, int WGN, int WGK, int MF, int NST, int BSRC = BSRC_PLAIN>
struct IgemmCfg {
    enum {
        NW    = WGM * WGN * WGK,                   // waves per workgroup
        NT    = NW * 64,
        NCH   = BKB / 16,                          // 16-byte chunks per row per step
        WTM   = BM / WGM,  WTN = BN / WGN,
        TM    = WTM / MF,  TN  = WTN / MF,
        FW    = (DT == DT_FP8) ? 2 : 1,            // 16-byte chunks per lane and operand
        KSUBB = ((MF == 32) ? 32 : 64) * FW,       // reduction bytes per MFMA
        NKSUB = BKB / KSUBB,
        CPL   = KSUBB / 16,                        // 16-byte chunks per MFMA along k
        RPI   = 1024 / BKB,                        // tile rows filled by one wave-level DMA
        IA    = BM / RPI / NW,                     // DMA instructions per wave per step, A tile
        IB    = BN / RPI / NW,
        LPT   = IA + IB,
        STAGE_BYTES  = (BM + BN) * BKB,
        EDGE_BYTES   = (BSRC == BSRC_NCHWS || BSRC == BSRC_NCHWE) ? 1024 : 0,   // direct reads: first and last 16 bytes of the tensor
        RING_BYTES   = NST * STAGE_BYTES + EDGE_BYTES,
        REDUCE_BYTES = (WGK > 1) ? WGK * BM * BN * 4 : 0,
        SMEM_BYTES   = (RING_BYTES > REDUCE_BYTES) ? RING_BYTES : REDUCE_BYTES,
        // direct NCHW reads: a wave-level DMA instruction must cover whole channel rows of the B tile
        ESZ   = (DT == DT_F16 || DT == DT_BF16) ? 2 : 1,
        DIRECT = (BSRC == BSRC_NCHW || BSRC == BSRC_NCHWS || BSRC == BSRC_NCHWE) ? 1 : 0,
        ROWS_OK = !DIRECT || ((BN * ESZ / 16) <= 64 && 64 % (BN * ESZ / 16) == 0),
        FITS  = (SMEM_BYTES <= 160 * 1024) && ((NST - 1) * LPT <= 63) && ROWS_OK,   // LDS capacity, vmcnt range, row rule
    };
    static_assert(BM % (WGM * MF) == 0 && BN % (WGN * MF) == 0, "wave tiles must be whole MFMA tiles");
    static_assert(NKSUB % WGK == 0 && NKSUB >= WGK, "in-group split must divide the sub-steps");
    static_assert(BKB % KSUBB == 0 && 1024 % BKB == 0, "step must be whole MFMAs and divide a DMA block");
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tiles must split evenly into per-wave DMA blocks");
    static_assert((NW * RPI) % 16 == 0, "the row swizzle must not depend on the DMA instruction index");
    static_assert(NST >= 2, "at least double buffering");
};

template <int DT, int BM, int BN, int BKB, int WGM, int WGN, int WGK, int MF, int NST, int OCC, int BSRC, int EPI>
__global__ void __launch_bounds__(WGM * WGN * WGK * 64, OCC)
igemm_kernel(const IgemmArgs g)
{
    typedef IgemmCfg<DT, BM, BN, BKB, WGM, WGN, WGK, MF, NST, BSRC> C;
    static_assert(C::FITS, "tile does not fit the LDS or the vmcnt range in this mode");
    typedef Mma<DT, MF> M;
    typedef typename M::acc_t acc_t;
    typedef typename M::elem_t elem_t;
    typedef typename M::frag_t frag_t;
    constexpr int FW = M::FW;
    constexpr int NW = C::NW, NCH = C::NCH, TM = C::TM, TN = C::TN, IA = C::IA, IB = C::IB, RPI = C::RPI;
    constexpr bool CONV = (BSRC != BSRC_PLAIN);     // conv-style output indexing
    constexpr int ES = (DT == DT_F16 || DT == DT_BF16) ? 2 : 1;   // operand element bytes
    constexpr int EPC = 16 / ES;                    // elements per 16-byte chunk
    constexpr int CPR = BN * ES / 16;               // NCHW mode: 16-byte chunks per channel row of the B tile
    constexpr int CRPI = 64 / CPR;                  // NCHW mode: channel rows per DMA instruction
    // NCHW mode: the 16-byte pixel chunks of channel row r are stored XOR-swizzled by nchw_swz(r), so that the
    // rows a transposing read touches together (8 for 1-byte, 4 for 2-byte elements, two or four chunks each)
    // fall into distinct LDS banks whatever the row pitch
    constexpr int SWZ_UNIT = (ES == 1) ? 2 : 4;                             // chunks that must stay adjacent
    constexpr int SWZ_DIV  = (16 / CPR > 1) ? 16 / CPR : 1;
    constexpr int SWZ_ROWS = (ES == 1) ? 8 : 4;                             // rows one transposing read touches
    constexpr int SWZ_MOD  = (CPR / SWZ_UNIT < SWZ_ROWS) ? CPR / SWZ_UNIT : SWZ_ROWS;
    auto nchw_swz = [&](int r) { return SWZ_MOD > 1 ? SWZ_UNIT * ((r / SWZ_DIV) % SWZ_MOD) : 0; };

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
#ifdef UNIT_PROBE
    unsigned long long unit_pt[8] = {0, 0, 0, 0, 0, 0, 0, 0}, unit_pr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    unsigned unit_w_vm = 0, unit_w_bar = 0, unit_w_frag = 0, unit_n_steps = 0;
#endif
    UNIT_STAMP(0);

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform: keeps LDS addresses scalar
    // (opaque from here on: otherwise the compiler re-derives it, and everything computed from it, from the
    // thread id inside the step loop for the code after the loop -- half a dozen instructions per step)
    asm volatile("" : "+s"(wave_s));
    const int wave = wave_s;
    const int wk   = wave / (WGM * WGN);
    const int wm   = (wave % (WGM * WGN)) / WGN;
    const int wn   = wave % WGN;

    // ---- tile coordinates.  Workgroups are dealt round-robin to the 8 XCDs (each with
    // its own L2): give every XCD one contiguous run of the tile order, and walk that
    // order in bands of 8 row-tiles so the tiles resident together share A and B rows.
    const int tiles_m = (g.rows + BM - 1) / BM;
    const int tiles_img = (g.PQ + BN - 1) / BN;     // per-image tiling only
    constexpr bool NCHW1 = (BSRC == BSRC_NCHW || BSRC == BSRC_NCHWE);     // 1x1 direct read, without / with edge patch
    constexpr bool EDGE1 = (BSRC == BSRC_NCHWE);
    const bool per_img = (NCHW1 || BSRC == BSRC_NCHWS) && g.per_img;
    const int tiles_n = per_img ? tiles_img * g.nimg : (g.col_limit - g.col_base + BN - 1) / BN;
    const int ntiles  = tiles_m * tiles_n;
    int bid = blockIdx.x;
    {   // XCD x = bid % 8 receives workgroups x, x + 8, ...: they become one contiguous run of the tile order
        const int q8 = ntiles >> 3, r8 = ntiles & 7, x = bid & 7;
        bid = x * q8 + (x < r8 ? x : r8) + (bid >> 3);
    }
    int tm, tn;
    if (g.row_runs) {
        // far more A (weight) bytes than B bytes: a run walks the column tiles of one row tile, so each
        // XCD fetches its own rows of A once and only the small B is fetched by every XCD
        tm = divu(bid, g.dv_tiles_n);
        tn = bid - tm * tiles_n;
    } else {
        constexpr int BAND = 8;
        const int band      = divu(bid, g.dv_band);
        const int band_m0   = band * BAND;
        const int band_rows = (tiles_m - band_m0 < BAND) ? tiles_m - band_m0 : BAND;
        const int in_band   = bid - band * BAND * tiles_n;
        tn = div_any(in_band, band_rows);
        tm = band_m0 + in_band - tn * band_rows;
    }
    const int row0 = tm * BM;
    int col0 = g.col_base + tn * BN, col_end = g.col_limit;   // first column of the tile, end of its column range
    if (per_img) {
        const int img = divu(tn, g.dv_tiles_img);
        col0 = img * g.PQ + (tn - img * tiles_img) * BN;
        col_end = (img + 1) * g.PQ;
    }

    const int ksteps_total = (g.kchunks + NCH - 1) / NCH;
    const int ks_begin = blockIdx.z * g.ksteps_per_split;
    int ks_end = ks_begin + g.ksteps_per_split;
    if (ks_end > ksteps_total) ks_end = ksteps_total;
    // first reduction chunk this workgroup must not load: later tiles come back as zeros
    const int kend = (ks_end * NCH < g.kchunks) ? ks_end * NCH : g.kchunks;

    // ---- global -> LDS bookkeeping.  DMA instruction j of wave w fills tile rows
    // (j*NW + w)*RPI .. +RPI; lane L lands in row L/NCH, physical chunk L%NCH of that
    // block and therefore fetches the logical chunk cT = (L%NCH) ^ swz(row).  NW*RPI is a
    // multiple of the swizzle period, so cT is the same for every j.
    const int lr_blk = lane / NCH;                                  // row inside a DMA block
    const int cT = (lane % NCH) ^ swz<NCH>(wave * RPI + lr_blk);    // logical chunk this thread fetches
    const int rows_here = (g.rows - row0 < BM) ? g.rows - row0 : BM;
    const __amdgpu_buffer_rsrc_t rsA =
        make_rsrc(g.A + (long)row0 * g.lda, (unsigned)((long)(rows_here - 1) * g.lda + (long)g.kchunks * 16));
    unsigned offA[IA];
#pragma unroll
    for (int j = 0; j < IA; ++j) {
        int r = (j * NW + wave) * RPI + lr_blk;
        offA[j] = (r < rows_here) ? (unsigned)(r * (int)g.lda + cT * 16) : UNIT_OOB;
    }
    const int cols_here = (col_end - col0 < BN) ? col_end - col0 : BN;
    const __amdgpu_buffer_rsrc_t rsB = (BSRC != BSRC_PLAIN)
        ? make_rsrc(g.B, (unsigned)g.b_bytes)
        : make_rsrc(g.B + (long)col0 * g.ldb, (unsigned)((long)(cols_here - 1) * g.ldb + (long)g.kchunks * 16));
    unsigned offB[IB];
    int bd0[IB], bh0[IB], bw0[IB];
#pragma unroll
    for (int j = 0; j < IB; ++j) {
        int r = (j * NW + wave) * RPI + lr_blk;
        bool valid = r < cols_here;
        if (BSRC == BSRC_NCHWS) {
            // lane -> (channel row inside the DMA block, 16-byte chunk of that row's window of pixels);
            // bd0 = byte offset of the chunk from the first byte the step needs of its first channel row
            // (a chunk of pixels lies inside one image, as in the 1x1 mode)
            const int crow = (j * NW + wave) * CRPI + lane / CPR;
            const int px = col0 + ((lane % CPR) ^ nchw_swz(crow)) * EPC;
            const int img = (g.cols > g.PQ) ? divu(px, g.dv_pq) : 0;
            bh0[j] = crow;
            bd0[j] = ((img * g.Cin + crow) * g.PQ + (px - img * g.PQ)) * ES;
            bw0[j] = 0;
            offB[j] = 0;
        } else if (NCHW1) {
            // lane -> (channel row inside the DMA block, 16-byte chunk of pixels)
            const int crow = (j * NW + wave) * CRPI + lane / CPR;
            // this lane's 16-byte chunk of pixels lies inside one image (the host only picks this
            // mode when the pixels per image are a multiple of the chunk); columns past the end
            // read whatever follows and are masked at the store
            const int px = col0 + ((lane % CPR) ^ nchw_swz(crow)) * EPC;
            const int img = (g.cols > g.PQ) ? divu(px, g.dv_pq) : 0;
            offB[j] = (unsigned)(((img * g.Cin + crow) * g.PQ + (px - img * g.PQ)) * ES);
            bh0[j] = crow;                          // channel row of this lane inside a step
            bd0[j] = bw0[j] = 0;
        } else if (BSRC == BSRC_GATHER || BSRC == BSRC_GATHERU) {
            int cc = valid ? col0 + r : 0;
            // (integer divisions are ~40 instructions each: skip the ones whose result is known)
            int n = 0, opq = cc;
            if (g.cols > g.PQ) { n = divu(cc, g.dv_pq); opq = cc - n * g.PQ; }   // more than one image
            int o = 0, pq = opq;
            if (g.PQ > g.P * g.Q) { o = divu(opq, g.dv_ppq); pq = opq - o * (g.P * g.Q); }   // output depth > 1
            int p = divu(pq, g.dv_q), q = pq - p * g.Q;
            // an invalid column gets a row far outside the image: its bounds test always fails
            const int bd = o * g.sd - g.pd, bh = p * g.sh - g.ph, bw = q * g.sw - g.pw;
            bd0[j] = bd;
            bh0[j] = valid ? bh : -0x100000;
            bw0[j] = bw;
            // byte offset of tap (0,0,0); modulo 2^32 (negative in the padding), exact once a tap is in range
            offB[j] = (unsigned)(((n * g.D + bd) * g.H + bh) * g.W + bw) * (unsigned)(g.CB * 16);
        } else {
            offB[j] = valid ? (unsigned)(r * (int)g.ldb + cT * 16) : UNIT_OOB;
            bd0[j] = bh0[j] = bw0[j] = 0;
        }
    }
    // conv: reduction chunk kc -> (r, s, channel chunk cb), advanced incrementally per step
    int kc = ks_begin * NCH + cT;
    int ct = 0, cr = 0, cs = 0, ccb = 0;
    constexpr bool uni_tap = (BSRC == BSRC_GATHERU);
    if (BSRC == BSRC_GATHER) {
        int trs = divu(kc, g.dv_cb);
        ccb = kc - trs * g.CB;
        int tr = divu(trs, g.dv_s);                 // tap rows from the start (over all planes)
        cs = trs - tr * g.S;
        ct = divu(tr, g.dv_r);
        cr = tr - ct * g.R;
    }

    // Gather fast path: when the channel chunks of a pixel are a whole number of steps
    // (CB % NCH == 0) every lane of a step works on the same tap, so the tap walk is scalar:
    // (ut, ur, us) and the byte offset `utap` of (tap, first chunk of the step) inside the packed
    // tensor.  Consecutive chunks are consecutive in memory across the s axis, so utap only
    // jumps when a tap row or plane ends.
    int ut = 0, ur = 0, us = 0, ucb = 0;
    unsigned utap = 0;
    if (uni_tap) {
        if (ks_begin != 0) {                    // only the later slices of a split reduction
            const int chunk0 = ks_begin * NCH;
            const int trs = chunk0 / g.CB;
            ucb = chunk0 - trs * g.CB;
            ut = trs / (g.R * g.S);
            const int rs = trs - ut * (g.R * g.S);
            ur = rs / g.S;
            us = rs - ur * g.S;
            utap = (unsigned)(((ut * g.H + ur) * g.W + us) * g.CB + ucb) * 16u;
        }
#pragma unroll
        for (int j = 0; j < IB; ++j) offB[j] += (unsigned)cT * 16u;   // this lane's chunk inside the step
    }

    // shifted direct read: (tap row, tap column, first channel chunk) of the step being issued and of
    // the step being read; wave-uniform, a step never straddles two taps (host-checked)
    int it_r = 0, it_s = 0, it_cb = 0, rt_r = 0, rt_s = 0, rt_cb = 0;
    if (BSRC == BSRC_NCHWS && ks_begin != 0) {
        const int chunk0 = ks_begin * NCH;
        const int tap = chunk0 / g.CB;
        it_cb = rt_cb = chunk0 - tap * g.CB;
        it_r = rt_r = tap / g.S;
        it_s = rt_s = tap - it_r * g.S;
    }
    // (the divisions above leave their results in vector registers; the tap walk is scalar work)
    it_r = rt_r = __builtin_amdgcn_readfirstlane(it_r);
    it_s = rt_s = __builtin_amdgcn_readfirstlane(it_s);
    it_cb = rt_cb = __builtin_amdgcn_readfirstlane(it_cb);
    if (EDGE1) rt_cb = ks_begin * NCH;  // 1x1 mode: first reduction chunk of the step being read
    int it_base = ((it_r - g.ph) * g.W + (it_s - g.pw)) * ES, it_cbo = it_cb * EPC * ES * g.PQ;

    // issues the DMA of the next tile (the one whose chunk for this thread is kc) into `stage`
    auto issue_tile = [&](int stage) {
        const bool kok = kc < kend;
        const unsigned kbyte = (unsigned)(kc - cT) * 16u;          // = step * BKB
        uint8_t *dst = smem + stage * C::STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int j = 0; j < IA; ++j)
            dma16(rsA, dst + j * NW * 1024, kok ? offA[j] + kbyte : UNIT_OOB);
        dst += BM * BKB;
        if (BSRC == BSRC_NCHWS) {
            // first byte this step needs of channel row 0 of its block: pixel col0 + delta of channel
            // it_cb*EPC.  The loads start at any byte, so every channel row lands with its window of
            // pixels at the tile's own columns.  A chunk that is not wholly inside the tensor comes back
            // as zeros: the few real pixels it holds (first and last channel only) are patched at the read
            // (it_base: byte offset of the tap, recomputed when the tap changes; it_cbo: of the channel block)
            const int base = it_base + it_cbo;
            const bool step_ok = (kc - cT) < kend;
#pragma unroll
            for (int j = 0; j < IB; ++j) {
                const int off = base + bd0[j];
                const bool ok = step_ok && off >= 0 && off + 16 <= (int)g.b_bytes;
                dma16(rsB, dst + j * NW * 1024, ok ? (unsigned)off : UNIT_OOB);
            }
            it_cb += NCH;
            it_cbo += NCH * EPC * ES * g.PQ;
            if (it_cb >= g.CB) {
                it_cb = 0;
                it_cbo = 0;
                if (++it_s == g.S) { it_s = 0; ++it_r; }
                it_base = ((it_r - g.ph) * g.W + (it_s - g.pw)) * ES;
            }
        } else if (NCHW1) {
            // channel rows of this step: chan0 .. chan0 + BKB/ES; rows past the real channel
            // count or past the slice end come back as zeros
            const int chan0 = (kc - cT) * EPC;
            const int chan_end = (kend * EPC < g.Cin) ? kend * EPC : g.Cin;
            // (edge variant: a chunk that is not wholly inside the tensor is not loaded: see read_frags)
            const unsigned lim = EDGE1 ? (unsigned)g.b_bytes : 0xffffffffu;
#pragma unroll
            for (int j = 0; j < IB; ++j) {
                const unsigned off = offB[j] + (unsigned)(chan0 * g.PQ * ES);
                const bool ok = chan0 + bh0[j] < chan_end && off + 16u <= lim;
                dma16(rsB, dst + j * NW * 1024, ok ? off : UNIT_OOB);
            }
        } else if (BSRC == BSRC_GATHERU) {
            const bool step_ok = (kc - cT) < kend;
#pragma unroll
            for (int j = 0; j < IB; ++j) {
                const int dd = bd0[j] + ut, h = bh0[j] + ur, w = bw0[j] + us;
                const bool ok = step_ok & ((unsigned)dd < (unsigned)g.D) & ((unsigned)h < (unsigned)g.H) &
                                ((unsigned)w < (unsigned)g.W);
                dma16(rsB, dst + j * NW * 1024, ok ? offB[j] + utap : UNIT_OOB);
            }
            ucb += NCH;
            utap += NCH * 16u;
            if (ucb >= g.CB) {
                ucb = 0;
                if (++us == g.S) {
                    us = 0;
                    utap += (unsigned)((g.W - g.S) * g.CB) * 16u;
                    if (++ur == g.R) {
                        ur = 0;
                        ++ut;
                        utap += (unsigned)((g.H - g.R) * g.W * g.CB) * 16u;
                    }
                }
            }
        } else if (BSRC == BSRC_GATHER) {
            const unsigned tap = (unsigned)(((ct * g.H + cr) * g.W + cs) * g.CB + ccb) * 16u;
#pragma unroll
            for (int j = 0; j < IB; ++j) {
                const int dd = bd0[j] + ct, h = bh0[j] + cr, w = bw0[j] + cs;
                const bool ok = kok & ((unsigned)dd < (unsigned)g.D) & ((unsigned)h < (unsigned)g.H) &
                                ((unsigned)w < (unsigned)g.W);
                dma16(rsB, dst + j * NW * 1024, ok ? offB[j] + tap : UNIT_OOB);
            }
            // whole taps to move on by (several when a pixel holds fewer chunks than a step), then whole tap rows
            // and planes: three divisions by reciprocal multiplies, no branches (per-lane loops here cost the
            // network stems a fifth of their step)
            ccb += NCH;
            const int adv = divu(ccb, g.dv_cb);
            ccb -= adv * g.CB;
            cs += adv;
            const int qs = divu(cs, g.dv_s);
            cs -= qs * g.S;
            cr += qs;
            const int qr = divu(cr, g.dv_r);
            cr -= qr * g.R;
            ct += qr;
        } else {
#pragma unroll
            for (int j = 0; j < IB; ++j)
                dma16(rsB, dst + j * NW * 1024, kok ? offB[j] + kbyte : UNIT_OOB);
        }
        kc += NCH;
    };

    // ---- fragment addressing (lane -> row inside an MFMA tile, 16-byte chunk along k)
    const int lrow   = lane % MF;
    const int lchunk = (lane / MF) * FW;            // first of this lane's FW chunks inside one MFMA
    const int a_row  = wm * C::WTM + lrow;
    const int b_row  = wn * C::WTN + lrow;
    const int a_swz  = swz<NCH>(a_row);             // unchanged by +MF*i (multiples of 16)
    const int b_swz  = swz<NCH>(b_row);
    // shifted direct read: image coordinates of this lane's output pixels (columns past the end
    // get a row outside the image, so every tap is masked)
    int sp[TN], sq[TN];
    if (BSRC == BSRC_NCHWS) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col0 + b_row + j * MF;
            const int pin = (g.cols > g.PQ) ? col - divu(col, g.dv_pq) * g.PQ : col;    // pixel inside its image
            const int p = divu(pin, g.dv_w);
            sp[j] = (col < col_end) ? p : -0x100000;
            sq[j] = pin - p * g.W;
        }
    }
    // Shifted direct read, per tap of the step being read (recomputed only when the tap changes; these loops are
    // bound by instruction issue): pixel index of tile column 0 in the first image, whether this wave may have to
    // patch the chunk that straddles the tensor's start / end, and the border mask of this lane's pixels.
    int r_wstart = 0;
    bool r_ns = false, r_ne = false, r_in[TN];
    auto reader_tap = [&]() {
        const int dr = rt_r - g.ph, dc = rt_s - g.pw;
        r_wstart = col0 + dr * g.W + dc;
        r_ns = wk == 0 && r_wstart < 0;
        r_ne = wk == WGK - 1 && r_wstart - (g.cols - g.PQ) + BN > g.PQ;
#pragma unroll
        for (int j = 0; j < TN; ++j)
            r_in[j] = (unsigned)(sp[j] + dr) < (unsigned)g.H && (unsigned)(sq[j] + dc) < (unsigned)g.W;
    };
    if (BSRC == BSRC_NCHWS) reader_tap();
    auto advance_reader = [&]() {
        rt_cb += NCH;
        if (rt_cb >= g.CB) {
            rt_cb = 0;
            if (++rt_s == g.S) { rt_s = 0; ++rt_r; }
            reader_tap();
        }
    };

    // ---- epilogue bookkeeping.  The unit of work of the epilogue is a GROUP: accumulator elements
    // 4a..4a+3 of one MFMA tile, which a lane holds for four consecutive rows of its column.  With an
    // in-group reduction split (WGK > 1) a wave owns every WGK-th group of its window (see the
    // reduction below), otherwise the groups of its own accumulators, one MFMA tile at a time.
    constexpr int NA = M::NACC, GPT = NA / 4;       // groups per MFMA tile
    constexpr int NG = TM * TN * GPT;               // groups per wave window
    static_assert(NG % WGK == 0 || NG < WGK, "the groups of a window must split evenly over its waves");
    // (a window with fewer groups than waves -- one 16x16 MFMA tile under a four-way split -- is finished by its first NG waves)
    constexpr int UG = (WGK > 1) ? (NG + WGK - 1) / WGK : GPT;  // groups handled together (their loads are issued first)
    constexpr int NU = (WGK > 1) ? 1 : TM * TN;     // such units per wave
    // first row (of four), column, and offset of (row 0, column) in the output of group q of unit u
    auto group_at = [&](int u, int q, int &grow, int &gcol, long &gcb) {
        const int gidx = (WGK > 1) ? q * WGK + wk : u * GPT + q;
        const int a4 = gidx % GPT, ij = gidx / GPT;
        const int j = ij % TN, i = ij / TN;
        grow = row0 + wm * C::WTM + i * MF + acc_row<MF>(4 * a4, lane);
        gcol = col0 + wn * C::WTN + j * MF + lrow;
        if (CONV) {
            const int n = (g.cols > g.cols_per_img) ? divu(gcol, g.dv_cpi) : 0;
            gcb = (long)n * g.img_stride + (gcol - n * g.cols_per_img);
        } else {
            gcb = gcol;
        }
    };
    // Requantise inputs of one unit (scale, bias, both residual forms), all through buffer descriptors:
    // absent inputs get an empty range and masked lanes an offset beyond it, both read as zero, so the
    // loads need no branches and the wave waits once for all of them.
    auto requant_inputs = [&](int u, float (*sc)[4], unsigned (*add)[4], unsigned *res4) {
        const __amdgpu_buffer_rsrc_t rsS = make_rsrc(g.scale, UNIT_OOB);
        const __amdgpu_buffer_rsrc_t rsBi = make_rsrc(g.bias, g.bias ? UNIT_OOB : 0u);
        const __amdgpu_buffer_rsrc_t rsR = make_rsrc(g.residual, g.residual ? UNIT_OOB : 0u);
        const __amdgpu_buffer_rsrc_t rsP = make_rsrc(g.res_packed, g.res_packed ? UNIT_OOB : 0u);
#pragma unroll
        for (int q = 0; q < UG; ++q) {
            int grow, gcol;
            long gcb;
            group_at(u, q, grow, gcol, gcb);
            const bool col_ok = gcol < col_end;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int row = grow + b;
                const unsigned off = row < g.rows ? (unsigned)row * 4u : UNIT_OOB;
                const unsigned roff = (row < g.rows && col_ok) ? (unsigned)(gcb + (long)row * g.row_stride) * 4u : UNIT_OOB;
                sc[q][b] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsS, off, 0, 0));
                add[q][b] = __builtin_amdgcn_raw_buffer_load_b32(rsBi, off, 0, 0) +
                            __builtin_amdgcn_raw_buffer_load_b32(rsR, roff, 0, 0);
            }
            // the four rows of a group are four consecutive output channels of the lane's pixel: the
            // packed residual arrives as one 32-bit load
            res4[q] = __builtin_amdgcn_raw_buffer_load_b32(
                rsP, (grow < g.packed_ld && col_ok) ? (unsigned)((long)gcol * g.packed_ld + grow) : UNIT_OOB, 0, 0);
        }
    };
    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < M::NACC; ++e) acc[i][j][e] = 0;

    // ---- main loop.  NST LDS stages hold the tile being multiplied and the NST-1 tiles
    // after it, which stream in by DMA while the MFMAs run.  Per step a wave runs NS
    // sub-steps; sub-step s issues the fragment reads of sub-step s+1 into the other half
    // of the fragment double buffer, then its own MFMAs.  The step's single barrier sits in
    // front of the LAST sub-step's MFMAs: after it the freed stage is re-armed with the
    // tile NST steps ahead and the first fragments of the next tile are read, so those
    // MFMAs cover barrier skew and LDS latency.
    constexpr int NS = C::NKSUB / WGK;              // sub-steps per wave per step
    // Small wave tiles (at most 4 MFMAs per sub-step) cannot hide an LDS read behind one
    // sub-step's MFMAs, so they keep whole steps in registers instead: while the MFMAs of step
    // ks run, all fragments of step ks+1 are read into the other register set (slots
    // set*NS + sub), and the step loop is unrolled by two so that the set is a constant.
    // The DMA then runs NST-1 tiles ahead and refills the stage read one step EARLIER (whose
    // reads every wave has consumed in its previous step's MFMAs), so the step's barrier needs
    // no wait on outstanding LDS reads: they complete behind the MFMAs and the DMA issue.
    constexpr bool WHOLE = (TM * TN <= 4) && NST >= 3;      // (the register-prefetch schedule needs three LDS stages)
    constexpr int NSLOT = WHOLE ? 2 * NS : 2;
    frag_t fa[NSLOT][TM], fb[NSLOT][TN];
    // The direct modes issue their transposing reads as inline assembly (see lds_tr), except in the kernels with the
    // highest register pressure (32-byte fragments on the large wave tiles): a fragment the compiler spilled or
    // moved between such a read and the kernel's own wait would be saved before it has arrived, so those keep the
    // builtins and the compiler's conservative waits.
    constexpr bool ASM_TR = !(FW == 2 && TM * TN >= 8);
    // Results of those reads stay in the 8-byte pieces the instructions return until the kernel has waited for them
    // (finish_frags): only then are they assembled into fragments, so that no register copy the compiler may need
    // for the assembly can run ahead of the data.
    v2i fbr[NSLOT][TN][2 * FW];
    // Shifted direct read: what remains to be done to the B fragments of a slot when they are used (border mask,
    // edge elements).  It is applied then and not at the read, so that nothing waits for the LDS data early.
    bool b_in[NSLOT][TN], b_fs[NSLOT][TN], b_fe[NSLOT][TN];
    unsigned b_vs[NSLOT][TN], b_ve[NSLOT][TN];
    auto finish_frags = [&](int slot) {
        if (!NCHW1 && BSRC != BSRC_NCHWS) return;
        if (ASM_TR) {
            UNIT_WAIT_LGKM0();                                  // (the transposing reads: see lds_tr)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                unsigned w[4 * FW];
#pragma unroll
                for (int h = 0; h < 2 * FW; ++h) {
                    lds_tr_done(fbr[slot][j][h]);
                    w[2 * h] = (unsigned)fbr[slot][j][h][0];
                    w[2 * h + 1] = (unsigned)fbr[slot][j][h][1];
                }
                fb[slot][j] = Frag<FW>::pack(w);
            }
        }
        constexpr bool TAPS = (BSRC == BSRC_NCHWS);
        if (!TAPS && !EDGE1) return;
        constexpr unsigned EMASK = (ES == 1) ? 0xffu : 0xffffu;
        constexpr int SH = 32 - 8 * ES;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            frag_t f = fb[slot][j];
            // (selects, no branches: the MFMA schedule wants one basic block per step)
            if (TAPS) f[0] = b_fs[slot][j] ? (int)(((unsigned)f[0] & ~EMASK) | b_vs[slot][j]) : f[0];
            f[4 * FW - 1] = b_fe[slot][j] ? (int)(((unsigned)f[4 * FW - 1] & ~(EMASK << SH)) | (b_ve[slot][j] << SH))
                                          : f[4 * FW - 1];
            if (TAPS) {
#pragma unroll
                for (int t = 0; t < 4 * FW; ++t) f[t] = b_in[slot][j] ? f[t] : 0;
            }
            fb[slot][j] = f;
        }
    };
    auto read_frags = [&](int stage, int sub, int slot) {
        const uint8_t *sA = smem + stage * C::STAGE_BYTES;
        const uint8_t *sB = sA + BM * BKB;
        const int ch = (sub * WGK + wk) * C::CPL + lchunk;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[slot][i] = Frag<FW>::load(sA + (a_row + i * MF) * BKB, ch, a_swz);
        if (DT == DT_U8A) {
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[slot][i] ^= (int)0x80808080;
        }
        if (NCHW1 || BSRC == BSRC_NCHWS) {
            // B tile is [channel][pixel], i.e. reduction-major: the transposing LDS reads of gfx950
            // hand every lane the 8 bytes of consecutive channels of its pixel column.  Within a group
            // of 16 lanes, lane t supplies the address of 8 contiguous bytes and lane n receives
            //   1-byte elements: byte n%8 of the rows supplied by lanes 2i + n/8,   i = 0..7
            //   2-byte elements: element n%4 of the rows supplied by lanes n/4 + 4i, i = 0..3
            // so lanes (2i, 2i+1) point at channel row i, pixels 0-7 and 8-15 of the group's 16 pixels
            // (four lanes per row, four pixels each, for 2-byte elements).
            constexpr int RPR = (ES == 1) ? 8 : 4;                  // channel rows per read
            const int t16 = lane & 15;
            const int trow = (ES == 1) ? (t16 >> 1) : (t16 >> 2);   // channel row this lane points at
            const int tcol = (ES == 1) ? (t16 & 1) * 8 : (t16 & 3) * 4;
            const int ncol = ((lane % MF) & ~15) + tcol;            // pixel inside the MFMA tile
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                unsigned w[4 * FW];
#pragma unroll
                for (int f = 0; f < FW; ++f) {
                    const int cbyte = (wn * C::WTN + j * MF + ncol) * ES;           // logical byte column of the row
                    const uint8_t *src = sB + ((ch + f) * EPC + trow) * (BN * ES) +
                                         ((((cbyte >> 4) ^ nchw_swz(trow)) << 4) | (cbyte & 15));
                    static_assert(EPC / RPR == 2, "two transposing reads per 16-byte fragment chunk");
                    v2i r0, r1;
                    if (ASM_TR) {
                        const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) const uint8_t *)src;
                        fbr[slot][j][2 * f] = lds_tr<ES, 0>(lds_addr);
                        fbr[slot][j][2 * f + 1] = lds_tr<ES, RPR * BN * ES>(lds_addr);
                        continue;
                    } else {
                        typedef __attribute__((address_space(3))) v2i lds_v2i;
                        typedef __attribute__((address_space(3))) v4s lds_v4s;
                        if (ES == 1) {
                            r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)src);
                            r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(src + RPR * BN * ES));
                        } else {
                            r0 = __builtin_bit_cast(v2i, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s *)src));
                            r1 = __builtin_bit_cast(v2i, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s *)(src + RPR * BN * ES)));
                        }
                    }
                    w[4 * f + 0] = (unsigned)r0[0];
                    w[4 * f + 1] = (unsigned)r0[1];
                    w[4 * f + 2] = (unsigned)r1[0];
                    w[4 * f + 3] = (unsigned)r1[1];
                }
                if (BSRC == BSRC_NCHWS || EDGE1) {
                    // shifted read: channel row c of the step holds pixels col0 + delta .. of its channel,
                    // delta = the tap's offset in the flattened image (0 in the 1x1 mode).  The tensor's start can
                    // only be straddled in the first image, where columns are pixel indices; its end in the last
                    constexpr bool TAPS = (BSRC == BSRC_NCHWS);
                    const int wstart = TAPS ? r_wstart : col0;          // pixel index of tile column 0 (first image)
                    const int m = wn * C::WTN + j * MF + lrow;          // this lane's tile column
                    const int pix = wstart + m, cstart = wstart + (m & ~(EPC - 1));
                    const uint8_t *edge = smem + NST * C::STAGE_BYTES;
                    // The chunk that straddles the start of the tensor was not loaded: its pixels of the
                    // first channel come from the tensor's first 16 bytes (kept at edge[0..15]) ...
                    b_fs[slot][j] = b_fe[slot][j] = false;
                    b_vs[slot][j] = b_ve[slot][j] = 0;
                    // (both cases are rare and wave-uniform: a scalar branch keeps them out of the other steps)
                    if (TAPS && sub == 0 && r_ns && rt_cb == 0) {
                        const bool fix = lchunk == 0 && cstart < 0 && pix >= 0;
                        const uint8_t *src = edge + (fix ? pix * ES : 0);
                        b_vs[slot][j] = (ES == 1) ? *src : *reinterpret_cast<const uint16_t *>(src);
                        b_fs[slot][j] = fix;
                    }
                    // ... and likewise the chunk that straddles its end, for the last channel (edge[16..31])
                    const int last0 = g.cols - g.PQ;                    // first column of the last image
                    const bool near_end = TAPS ? (r_ne && rt_cb + NCH >= g.CB)
                                               : (wk == WGK - 1 && rt_cb + NCH >= g.kchunks && wstart - last0 + BN > g.PQ);
                    if (sub == NS - 1 && near_end) {
                        const int pixl = pix - last0, cstartl = cstart - last0;
                        const bool fix = lchunk == C::CPL - FW && cstartl + EPC > g.PQ && pixl < g.PQ;
                        const uint8_t *src = edge + 16 + (fix ? (pixl - (g.PQ - EPC)) * ES : 0);
                        b_ve[slot][j] = (ES == 1) ? *src : *reinterpret_cast<const uint16_t *>(src);
                        b_fe[slot][j] = fix;
                    }
                    // taps that fall into the padding (or columns past the image) contribute zero
                    if (TAPS) b_in[slot][j] = r_in[j];
                }
                if (!ASM_TR) fb[slot][j] = Frag<FW>::pack(w);   // (otherwise assembled in finish_frags)
            }
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[slot][j] = Frag<FW>::load(sB + (b_row + j * MF) * BKB, ch, b_swz);
        }
        if (DT == DT_U8B) {
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[slot][j] ^= (int)0x80808080;
        }
    };

    if (ks_begin < ks_end) {
        constexpr int AHEAD = WHOLE ? NST - 1 : NST;            // tiles in flight after the prologue
        if ((BSRC == BSRC_NCHWS || EDGE1) && wave == 0)   // first and last 16 bytes of the tensor (see read_frags)
            dma16(rsB, smem + NST * C::STAGE_BYTES,
                  lane == 0 ? 0u : lane == 1 ? (unsigned)(g.b_bytes - 16) : UNIT_OOB);
        UNIT_STAMP(6);
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) issue_tile(t);          // (zeros past the slice end)
        UNIT_STAMP(7);
        UNIT_WAIT_VM_LGKM0((AHEAD - 1) * C::LPT);               // own part of tile 0 has landed
        UNIT_BARRIER();
        UNIT_STAMP(1);
        int stage = 0;
        if (WHOLE) {
#pragma unroll
            for (int s2 = 0; s2 < NS; ++s2) read_frags(0, s2, s2);
            // The step loop is unrolled over the fragment sets and the stage ring (four steps), so that set and
            // stages are constants: LDS addresses fold into the instructions' offsets and the ring arithmetic
            // disappears.  These loops run one wave per SIMD and are bound by instruction issue.
            static_assert(!WHOLE || NST == 4, "the unrolled step loop walks a ring of four stages");
            auto whole_step = [&](auto set_c, auto stage_c) {
                constexpr int SET = decltype(set_c)::value;
                constexpr int STG = decltype(stage_c)::value;
                constexpr int next_stage = (STG + 1) % NST;
                constexpr int prev_stage = (STG + NST - 1) % NST;
#ifdef UNIT_PROBE
                const unsigned unit_c0 = UNIT_CYC();
#endif
                UNIT_WAIT_VM((NST >= 3 ? NST - 3 : 0) * C::LPT);   // own part of the next tile has landed
#ifdef UNIT_PROBE
                const unsigned unit_c1 = UNIT_CYC();
#endif
                UNIT_BARRIER();
#ifdef UNIT_PROBE
                const unsigned unit_c2 = UNIT_CYC();
#endif
#pragma unroll
                for (int s2 = 0; s2 < NS; ++s2) finish_frags(SET * NS + s2);   // (read one step ago)
#ifdef UNIT_PROBE
                const unsigned unit_c3 = UNIT_CYC();
                UNIT_ACC(unit_w_vm, unit_c0, unit_c1);  UNIT_ACC(unit_w_bar, unit_c1, unit_c2);
                UNIT_ACC(unit_w_frag, unit_c2, unit_c3);  ++unit_n_steps;
#endif
                __builtin_amdgcn_sched_barrier(0);
                if (BSRC == BSRC_NCHWS) advance_reader();
                if (EDGE1) rt_cb += NCH;
#pragma unroll
                for (int s2 = 0; s2 < NS; ++s2) read_frags(next_stage, s2, (SET ^ 1) * NS + s2);
                issue_tile(prev_stage);                          // tile ks+NST-1 into the stage read one step ago
#pragma unroll
                for (int s2 = 0; s2 < NS; ++s2)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            M::run(acc[i][j], fa[SET * NS + s2][i], fb[SET * NS + s2][j]);
                {
                    // the reads go first (their data is due one step later), then the DMAs are
                    // spread between the MFMAs
                    constexpr int NMFMA = NS * TM * TN;
                    constexpr int VPM = (C::LPT + NMFMA - 1) / NMFMA;
                    __builtin_amdgcn_sched_group_barrier(0x100, NS * (TM + TN) * FW, 0);
#pragma unroll
                    for (int r = 0; r < NMFMA; ++r) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // MFMA
                        __builtin_amdgcn_sched_group_barrier(0x020, VPM, 0);    // global -> LDS DMA
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            // (whole rounds of the ring in a loop with a single exit, then the remaining steps: a loop with an
            // exit after every step makes the compiler carry an exit flag and placeholder copies through each step)
            int steps_left = ks_end - ks_begin;
            for (; steps_left >= 4; steps_left -= 4) {
                whole_step(IntC<0>{}, IntC<0>{});
                whole_step(IntC<1>{}, IntC<1>{});
                whole_step(IntC<0>{}, IntC<2>{});
                whole_step(IntC<1>{}, IntC<3>{});
            }
            if (steps_left >= 1) whole_step(IntC<0>{}, IntC<0>{});
            if (steps_left >= 2) whole_step(IntC<1>{}, IntC<1>{});
            if (steps_left >= 3) whole_step(IntC<0>{}, IntC<2>{});
        } else {
        read_frags(0, 0, 0);
        for (int ks = ks_begin; ks < ks_end; ++ks) {
            const int next_stage = (stage + 1 == NST) ? 0 : stage + 1;
#pragma unroll
            for (int s2 = 0; s2 < NS; ++s2) {
                const int slot = s2 & 1;
                const bool last = (s2 + 1 == NS);
                if (last) {
                    UNIT_WAIT_VM_LGKM0((NST - 2) * C::LPT);     // next tile landed, my reads of this one done
                    UNIT_BARRIER();
                }
                finish_frags(slot);
                __builtin_amdgcn_sched_barrier(0);
                // One scheduling region: the MFMAs of this sub-step plus the memory
                // instructions that must be in flight before the next one -- the fragment
                // reads of the next sub-step and, after the barrier, the DMA that re-arms the
                // freed stage.  The group barriers below spread those between the MFMAs so
                // the matrix pipe never waits behind a burst of memory instructions.
                if (!last) {
                    read_frags(stage, s2 + 1, slot ^ 1);
                } else {
                    if (BSRC == BSRC_NCHWS) advance_reader();
                    if (EDGE1) rt_cb += NCH;
                    read_frags(next_stage, 0, slot ^ 1);
                    issue_tile(stage);                           // tile ks+NST into the stage just freed
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        M::run(acc[i][j], fa[slot][i], fb[slot][j]);
                {
                    constexpr int NMEM = (TM + TN) * FW + C::LPT;   // upper bound: reads + DMAs
                    constexpr int PER  = (TM * TN / NMEM) > 0 ? (TM * TN / NMEM) : 1;
#pragma unroll
                    for (int r = 0; r < (TM + TN) * FW; ++r) {
                        __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);   // MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // LDS read
                    }
                    if (last) {
#pragma unroll
                        for (int r = 0; r < C::LPT; ++r) {
                            __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);   // MFMA
                            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);     // global -> LDS DMA
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (NS & 1) {                            // odd sub-step count: next tile's first fragments sit in slot 1
                if (ASM_TR && (NCHW1 || BSRC == BSRC_NCHWS)) {   // (their transposing reads must have landed before they are copied)
                    UNIT_WAIT_LGKM0();
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int h = 0; h < 2 * FW; ++h) {
                            lds_tr_done(fbr[1][j][h]);
                            fbr[0][j][h] = fbr[1][j][h];
                        }
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[0][i] = fa[1][i];
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[0][j] = fb[1][j];
                if (BSRC == BSRC_NCHWS || EDGE1) {
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        b_in[0][j] = b_in[1][j];  b_fs[0][j] = b_fs[1][j];  b_fe[0][j] = b_fe[1][j];
                        b_vs[0][j] = b_vs[1][j];  b_ve[0][j] = b_ve[1][j];
                    }
                }
            }
            stage = next_stage;
        }
        }
        UNIT_STAMP(2);
        UNIT_WAIT_VM_LGKM0(0);                       // drain the (zero-fill) DMAs of the tiles past the end
        UNIT_BARRIER();
        UNIT_STAMP(3);
    }

    // ---- in-group split reduction and epilogue.  With an in-group reduction split every wave parks
    // all of its groups in LDS (16 bytes per lane, lane-contiguous, conflict free) and then adds the WGK
    // partial sums of the groups it owns in fixed order and runs the epilogue for them, so the reduction
    // and the epilogue are shared by all waves of the window instead of falling to one.
    typedef elem_t v4e __attribute__((ext_vector_type(4)));
    const v4e *red = reinterpret_cast<const v4e *>(smem);
    const int wmn = wave % (WGM * WGN);
    if (WGK > 1) {
        v4e *park = reinterpret_cast<v4e *>(smem);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int a4 = 0; a4 < GPT; ++a4)
                    park[((wk * WGM * WGN + wmn) * NG + (i * TN + j) * GPT + a4) * 64 + lane] =
                        v4e{acc[i][j][4 * a4], acc[i][j][4 * a4 + 1], acc[i][j][4 * a4 + 2], acc[i][j][4 * a4 + 3]};
        __syncthreads();
        if (NG < WGK && wk >= NG) return;           // (no barrier follows)
    }

    const elem_t *tile_base = reinterpret_cast<const elem_t *>(g.out) + (long)blockIdx.z * g.split_stride +
                              (long)row0 * g.row_stride;
    const __amdgpu_buffer_rsrc_t rsO = make_rsrc(tile_base, UNIT_OOB);        // raw stores; lanes are masked explicitly
    // unsigned-operand correction of the raw epilogue (added once, by the first reduction slice; the
    // per-row form is allocated in whole 256-byte blocks)
    const __amdgpu_buffer_rsrc_t rsFix = make_rsrc(
        g.bias, !(g.bias && blockIdx.z == 0) ? 0u : (DT == DT_U8B) ? (unsigned)((g.rows * 4 + 255) & ~255) : UNIT_OOB);
    elem_t *out = reinterpret_cast<elem_t *>(g.out);

#pragma clang loop unroll(full)
    for (int u = 0; u < NU; ++u) {
        v4e val[UG];
        int grow[UG], gcol[UG];
        long gcb[UG];
#pragma unroll
        for (int q = 0; q < UG; ++q) {
            group_at(u, q, grow[q], gcol[q], gcb[q]);
            if (WGK > 1) {
                const int gidx = q * WGK + wk;
                v4e v = red[((0 * WGM * WGN + wmn) * NG + gidx) * 64 + lane];
#pragma unroll
                for (int k2 = 1; k2 < WGK; ++k2) v += red[((k2 * WGM * WGN + wmn) * NG + gidx) * 64 + lane];
                val[q] = v;
            } else {
                // (u and q are unrolled constants here, so this indexes registers statically)
                val[q] = v4e{acc[u / TN][u % TN][4 * q], acc[u / TN][u % TN][4 * q + 1],
                             acc[u / TN][u % TN][4 * q + 2], acc[u / TN][u % TN][4 * q + 3]};
            }
        }
        if (EPI == EPI_RAW) {
            // 4-byte stores through a buffer descriptor anchored at the tile's first row; out-of-tile
            // lanes get an out-of-range offset and are dropped by the hardware.  Unsigned operands: per
            // column (DT_U8A) one correction for the group, per row (DT_U8B) one 16-byte load of four.
            v4i fix[UG];
#pragma unroll
            for (int q = 0; q < UG; ++q) {
                if (DT == DT_U8B) {
                    fix[q] = buf_load16(rsFix, (unsigned)grow[q] * 4u);
                } else if (DT == DT_U8A) {
                    const int f = (int)__builtin_amdgcn_raw_buffer_load_b32(rsFix, gcol[q] < col_end ? (unsigned)gcol[q] * 4u : UNIT_OOB, 0, 0);
                    fix[q] = v4i{f, f, f, f};
                } else {
                    fix[q] = v4i{0, 0, 0, 0};
                }
            }
#pragma unroll
            for (int q = 0; q < UG; ++q) {
                const unsigned cb = (unsigned)gcb[q];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int lr = grow[q] - row0 + b;
                    const bool ok = gcol[q] < col_end && lr < rows_here;
                    const unsigned off = ok ? (cb + (unsigned)lr * (unsigned)g.row_stride) * 4u : UNIT_OOB;
                    elem_t v = val[q][b];
                    if (DT == DT_U8A || DT == DT_U8B) v += (elem_t)fix[q][b];
                    __builtin_amdgcn_raw_buffer_store_b32(to_bits(v), rsO, off, 0, 0);
                }
            }
        } else {
            // every load of the unit is issued before its first store
            float sc[UG][4];
            unsigned add[UG][4], res4[UG];          // modular sums: the caller bounds only the total
            requant_inputs(u, sc, add, res4);
#pragma unroll
            for (int q = 0; q < UG; ++q) {
                if (gcol[q] >= col_end) continue;
                unsigned four = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int row = grow[q] + b;
                    if (row >= g.rows) continue;
                    const long addr = gcb[q] + (long)row * g.row_stride;
                    const int t = (int)((unsigned)(int)val[q][b] + add[q][b] +
                                        (unsigned)((int)(int8_t)(res4[q] >> (8 * b)) * g.res_mult));
                    if (g.store_raw) out[addr] = val[q][b];
                    const int v = requant_elem(t, sc[q][b], g.relu);
                    if (g.out_i8) g.out_i8[addr] = (int8_t)v;
                    four |= ((unsigned)v & 0xffu) << (8 * b);
                }
                // the int8 results of a group leave as one 32-bit store into the packed (NHWC) output
                // (padding channels stay zero)
                if (g.out_packed && grow[q] < g.packed_ld)
                    *reinterpret_cast<unsigned *>(g.out_packed + (long)gcol[q] * g.packed_ld + grow[q]) = four;
            }
        }
    }
#ifdef UNIT_PROBE
    UNIT_STAMP(4);
    if (g.probe) {
        __builtin_amdgcn_s_waitcnt(0);
        UNIT_STAMP(5);
        if (lane == 0) {
            unsigned long long *o = g.probe + ((size_t)blockIdx.x * NW + wave) * 16;
#pragma unroll
            for (int i = 0; i < 8; ++i) { o[i] = unit_pt[i];  o[8 + i] = unit_pr[i]; }
            // (cycle stamps 3-6 are not used by the readers: the step loop's wait sums go there)
            o[3] = unit_w_vm;  o[4] = unit_w_bar;  o[5] = unit_w_frag;  o[6] = unit_n_steps;
        }
    }
#endif
}

}  // namespace unit
