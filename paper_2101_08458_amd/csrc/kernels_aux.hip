// Layout packing, split-reduction epilogue and the small int8 network operators.
// All of them are bandwidth-bound permutations / elementwise passes.
#include "unit_internal.h"

namespace unit {

// ------------------------------------------------------------------ pack_act
// NCHW -> [n][h*w][cp] with cp = channels padded to 16 bytes (zero filled): the graph
// level layout change of the paper (Section V-C; Section II-C.1 for the padding) done as
// one tiled transpose through LDS.  T = int8_t (16 channels per chunk) or uint16_t (8).
// With Q > 0 only the pixels (p*srow_step, q*scol_step) of each input image are packed
// (HW = P*Q output pixels, HWin = pixels per input channel): the input of a strided 1x1 conv.
template <typename T>
__global__ void __launch_bounds__(256)
pack_act_kernel(const T *__restrict__ x, uint8_t *__restrict__ xp, int C, int HW, int cp,
                int HWin, int Q, int srow, int scol)
{
    constexpr int CH = 16 / sizeof(T);            // channels per 16-byte chunk
    constexpr int TP = 64;                        // pixels per tile
    constexpr int TC = 64;                        // channels per tile
    __shared__ T tile[TC][TP + 4 / sizeof(T)];
    const int tid = threadIdx.x;
    const int hw0 = blockIdx.x * TP, c0 = blockIdx.y * TC, n = blockIdx.z;
    const T *xn = x + (long)n * C * HWin;
    {
        const int px = tid & 63;
        int src = hw0 + px;
        if (Q > 0) {                               // subsampled source pixel
            const int p = src / Q;
            src = p * srow + (src - p * Q) * scol;
        }
        // every load is issued before the first LDS store: a masked element reads element 0 of
        // the image instead of branching around its load, and is zeroed afterwards
        const bool px_ok = hw0 + px < HW;
        T v[TC / 4];
#pragma unroll
        for (int i = 0; i < TC / 4; ++i) {
            const int c = (tid >> 6) + 4 * i;
            const bool ok = px_ok && c0 + c < C;
            v[i] = xn[ok ? (long)(c0 + c) * HWin + src : 0];
        }
#pragma unroll
        for (int i = 0; i < TC / 4; ++i) {
            const int c = (tid >> 6) + 4 * i;
            tile[c][px] = (px_ok && c0 + c < C) ? v[i] : (T)0;
        }
    }
    __syncthreads();
    constexpr int CHUNKS = TC / CH;               // chunks per pixel inside the tile
#pragma unroll
    for (int i = 0; i < TP * CHUNKS / 256; ++i) {
        int id = tid + i * 256;
        int px = id / CHUNKS, cc = id % CHUNKS;
        if (hw0 + px >= HW || c0 + cc * CH >= cp) continue;
        __attribute__((aligned(16))) T vals[CH];
#pragma unroll
        for (int e = 0; e < CH; ++e) vals[e] = tile[cc * CH + e][px];
        *reinterpret_cast<v4i *>(xp + (((long)n * HW + hw0 + px) * cp + c0 + cc * CH) * sizeof(T)) =
            *reinterpret_cast<const v4i *>(vals);
    }
}

// The same transpose with the two mechanisms of the main kernel's direct 1x1 read: the 64-channel x TP-pixel tile
// comes into LDS with 16-byte global -> LDS loads (any byte offset; a row of pixels per channel, chunks XOR-swizzled
// by row), and gfx950's transposing LDS reads hand every lane the 16 bytes of consecutive channels of its pixel, i.e.
// one chunk of the packed tensor (see read_frags in igemm.hpp for the lane layout).  Lanes 16g..16g+15 of a wave hold
// chunk g of 16 consecutive pixels, so a wave's store covers whole 64-byte runs of the packed rows.  ES = element
// bytes; TP is chosen so that a channel row of the tile is a whole 128-byte line.  Needs rows that start on dword boundaries (the range check of those loads works per dword) and a tensor
// below 2 GiB; the byte-wise kernel above takes the rest.
template <int ES, int TP>
__global__ void __launch_bounds__(256)
pack_act_tr_kernel(const uint8_t *__restrict__ x, uint8_t *__restrict__ xp, int C, int HW, int cp, unsigned x_bytes)
{
    constexpr int TC = 64;                        // channels per tile (TP pixels)
    constexpr int EPC = 16 / ES;                  // elements per 16-byte chunk
    constexpr int CPR = TP * ES / 16;             // chunks per channel row of the tile
    constexpr int CRPI = 64 / CPR;                // channel rows per wave-level load
    constexpr int NI = TC / CRPI / 4;             // loads per wave
    constexpr int RPR = (ES == 1) ? 8 : 4;        // channel rows per transposing read
    constexpr int SWZ_UNIT = (ES == 1) ? 2 : 4, SWZ_DIV = (16 / CPR > 1) ? 16 / CPR : 1;
    constexpr int SWZ_MOD = (CPR / SWZ_UNIT < RPR) ? CPR / SWZ_UNIT : RPR;
    static_assert(SWZ_DIV * SWZ_MOD == RPR, "the swizzle must repeat with the rows of one transposing read");
    auto swz = [](int r) { return SWZ_MOD > 1 ? SWZ_UNIT * ((r / SWZ_DIV) % SWZ_MOD) : 0; };
    __shared__ __attribute__((aligned(16))) uint8_t tile[TC * TP * ES];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hw0 = blockIdx.x * TP, c0 = blockIdx.y * TC, n = blockIdx.z;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(x, x_bytes);
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int crow = (j * 4 + wave) * CRPI + lane / CPR;
        const int px = hw0 + ((lane % CPR) ^ swz(crow)) * EPC;
        const int c = c0 + crow;
        // (channels past C read as zeros: the padding of the packed rows; pixels past the image are never stored)
        const unsigned off = c < C ? (unsigned)((((long)n * C + c) * HW + px) * ES) : UNIT_OOB;
        dma16(rs, tile + (j * 4 + wave) * 1024, off);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    const int t16 = lane & 15;
    const int trow = (ES == 1) ? (t16 >> 1) : (t16 >> 2);      // channel row this lane points at
    const int tcol = (ES == 1) ? (t16 & 1) * 8 : (t16 & 3) * 4;
#pragma unroll
    for (int pg = wave; pg < TP / 16; pg += 4) {               // groups of 16 pixels of the tile, dealt to the waves
    const int cbyte = (pg * 16 + tcol) * ES;
    const int px = hw0 + pg * 16 + t16;
#pragma unroll
    for (int it = 0; it < TC / EPC / 4; ++it) {
        const int cc = it * 4 + (lane >> 4);                   // chunk of the tile's channels
        const uint8_t *src = tile + (cc * EPC + trow) * (TP * ES) + ((((cbyte >> 4) ^ swz(trow)) << 4) | (cbyte & 15));
        typedef __attribute__((address_space(3))) v2i lds_v2i;
        typedef __attribute__((address_space(3))) v4s lds_v4s;
        v2i r0, r1;
        if (ES == 1) {
            r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)src);
            r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(src + RPR * TP * ES));
        } else {
            r0 = __builtin_bit_cast(v2i, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s *)src));
            r1 = __builtin_bit_cast(v2i, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s *)(src + RPR * TP * ES)));
        }
        if (px < HW && c0 + cc * EPC < cp)
            *reinterpret_cast<v4i *>(xp + (((long)n * HW + px) * cp + c0 + cc * EPC) * ES) = v4i{r0[0], r0[1], r1[0], r1[1]};
    }
    }
}

// Images whose channels fit one 16-byte chunk (network inputs): one thread per pixel reads its
// CL >= C channel values (coalesced along the pixels; channels past C re-read channel 0 and are
// zeroed) and writes the pixel's chunk.  The tiled transpose above would spend a 64-channel tile
// on them.
template <typename T, int CL>
__global__ void __launch_bounds__(256)
pack_act_smallc_kernel(const T *__restrict__ x, uint8_t *__restrict__ xp, int C, int HW,
                       int HWin, int Q, int srow, int scol)
{
    constexpr int CH = 16 / sizeof(T);
    const int px = blockIdx.x * 256 + threadIdx.x, n = blockIdx.y;
    if (px >= HW) return;
    int src = px;
    if (Q > 0) {
        const int p = px / Q;
        src = p * srow + (px - p * Q) * scol;
    }
    const T *xn = x + (long)n * C * HWin + src;
    __attribute__((aligned(16))) T vals[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) vals[c] = 0;
    T v[CL];
#pragma unroll
    for (int c = 0; c < CL; ++c) v[c] = xn[(long)(c < C ? c : 0) * HWin];
#pragma unroll
    for (int c = 0; c < CL; ++c) vals[c] = c < C ? v[c] : (T)0;
    *reinterpret_cast<v4i *>(xp + ((long)n * HW + px) * 16) = *reinterpret_cast<const v4i *>(vals);
}

template <typename T>
static void launch_pack_small(const T *x, uint8_t *xp, int n, int c, int hw, int hw_in, int Q, int srow, int scol,
                              hipStream_t st)
{
    const dim3 grid((hw + 255) / 256, n), block(256);
    if (c <= 4)
        hipLaunchKernelGGL((pack_act_smallc_kernel<T, 4>), grid, block, 0, st, x, xp, c, hw, hw_in, Q, srow, scol);
    else if (c <= 8 || sizeof(T) == 2)
        hipLaunchKernelGGL((pack_act_smallc_kernel<T, 8>), grid, block, 0, st, x, xp, c, hw, hw_in, Q, srow, scol);
    else
        hipLaunchKernelGGL((pack_act_smallc_kernel<T, 16 / sizeof(T)>), grid, block, 0, st, x, xp, c, hw, hw_in, Q, srow, scol);
}

// sh, sw > 1 with p, q > 0: pack only the pixels (i*sh, j*sw), i < p, j < q (output [n][p*q][cp])
hipError_t launch_pack_act_sub(int dtype, int n, int c, int h, int w, int sh, int sw, int p, int q,
                               const void *x, void *xp, hipStream_t st)
{
    const bool sub = p > 0;
    const int hw_in = h * w, hw = sub ? p * q : hw_in;
    const int Q = sub ? q : 0, srow = sh * w, scol = sw;
    const int chunk = (dtype == DT_I8) ? 16 : 8;
    if (c <= chunk && n <= 65535) {
        if (dtype == DT_I8) launch_pack_small((const int8_t *)x, (uint8_t *)xp, n, c, hw, hw_in, Q, srow, scol, st);
        else                launch_pack_small((const uint16_t *)x, (uint8_t *)xp, n, c, hw, hw_in, Q, srow, scol, st);
        return hipGetLastError();
    }
    const int es = (dtype == DT_I8) ? 1 : 2;
    const long x_bytes = (long)n * c * hw_in * es;
    if (!sub && ((long)hw * es) % 4 == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0 && x_bytes < (1L << 31)) {
        const int cp = (c + chunk - 1) / chunk * chunk;
        const int tp = 128 / es;                   // tile pixels: one 128-byte line per channel row
        dim3 grid((hw + tp - 1) / tp, (cp + 63) / 64, n);
        if (es == 1) hipLaunchKernelGGL((pack_act_tr_kernel<1, 128>), grid, dim3(256), 0, st, (const uint8_t *)x, (uint8_t *)xp, c, hw, cp, (unsigned)x_bytes);
        else         hipLaunchKernelGGL((pack_act_tr_kernel<2, 64>), grid, dim3(256), 0, st, (const uint8_t *)x, (uint8_t *)xp, c, hw, cp, (unsigned)x_bytes);
        return hipGetLastError();
    }
    if (dtype == DT_I8) {   // callers pass the storage type: one- or two-byte elements
        const int cp = (c + 15) / 16 * 16;
        dim3 grid((hw + 63) / 64, (cp + 63) / 64, n);
        hipLaunchKernelGGL(pack_act_kernel<int8_t>, grid, dim3(256), 0, st,
                           (const int8_t *)x, (uint8_t *)xp, c, hw, cp, hw_in, Q, srow, scol);
    } else {
        const int cp = (c + 7) / 8 * 8;
        dim3 grid((hw + 63) / 64, (cp + 63) / 64, n);
        hipLaunchKernelGGL(pack_act_kernel<uint16_t>, grid, dim3(256), 0, st,
                           (const uint16_t *)x, (uint8_t *)xp, c, hw, cp, hw_in, Q, srow, scol);
    }
    return hipGetLastError();
}

hipError_t launch_pack_act(int dtype, int n, int c, int h, int w, const void *x, void *xp, hipStream_t st)
{
    return launch_pack_act_sub(dtype, n, c, h, w, 1, 1, 0, 0, x, xp, st);
}

// packed int8 [n][hw][cp] -> NCHW
__global__ void unpack_act_i8_kernel(const int8_t *__restrict__ xp, int8_t *__restrict__ x,
                                     int C, int HW, int cp, long total)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int px = i % HW;
    long nc = i / HW;
    int c = nc % C;
    long n = nc / C;
    x[i] = xp[(n * HW + px) * cp + c];
}

hipError_t launch_unpack_act_i8(int n, int c, int h, int w, const void *xp, int8_t *x, hipStream_t st)
{
    long total = (long)n * c * h * w;
    int cp = (c + 15) / 16 * 16;
    hipLaunchKernelGGL(unpack_act_i8_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const int8_t *)xp, x, c, h * w, cp, total);
    return hipGetLastError();
}

// ------------------------------------------------------------------ pack_weights
// OIHW -> [k][r][s][cp]: each output channel's reduction becomes one contiguous,
// zero-padded row (the "column-major B" of the implicit GEMM).  Done once per layer.
template <typename T>
__global__ void pack_weights_kernel(const T *__restrict__ w, T *__restrict__ wp,
                                    int C, int RS, int cp, long total)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;   // index into wp
    if (i >= total) return;
    int c = i % cp;
    long t = i / cp;
    int rs = t % RS;
    long k = t / RS;
    wp[i] = (c < C) ? w[(k * C + c) * RS + rs] : (T)0;
}

hipError_t launch_pack_weights(int dtype, int k, int c, int r, int s, const void *w, void *wp, hipStream_t st)
{
    if (dtype == DT_I8) {   // callers pass the storage type: one- or two-byte elements
        int cp = (c + 15) / 16 * 16;
        long total = (long)k * r * s * cp;
        hipLaunchKernelGGL(pack_weights_kernel<int8_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const int8_t *)w, (int8_t *)wp, c, r * s, cp, total);
    } else {
        int cp = (c + 7) / 8 * 8;
        long total = (long)k * r * s * cp;
        hipLaunchKernelGGL(pack_weights_kernel<uint16_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const uint16_t *)w, (uint16_t *)wp, c, r * s, cp, total);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ pad_rows
// Copy a [rows][row_bytes] matrix (row pitch ld_bytes, any alignment) into a dense
// [rows][dst_row_bytes] one, zero filling the tail: matmul operands that do not meet the
// 16-byte rule of the main kernel.
__global__ void pad_rows_kernel(const uint8_t *__restrict__ src, long ld_bytes, int row_bytes,
                                uint8_t *__restrict__ dst, int dst_row_bytes, long total)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int b = i % dst_row_bytes;
    long r = i / dst_row_bytes;
    dst[i] = (b < row_bytes) ? src[r * ld_bytes + b] : (uint8_t)0;
}

hipError_t launch_pad_rows(const void *src, long ld_bytes, int rows, int row_bytes,
                           void *dst, int dst_row_bytes, hipStream_t st)
{
    long total = (long)rows * dst_row_bytes;
    hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t *)src, ld_bytes, row_bytes, (uint8_t *)dst, dst_row_bytes, total);
    return hipGetLastError();
}

// ------------------------------------------------------------------ split-K reduce + epilogue
// Sums the per-workgroup partial accumulators in slice order (fixed order: fp32 results
// are run-to-run identical), then applies the same epilogue as the main kernel.  The
// split reduction is the paper's "split reduction" tuning step (Section III-C.3) carried
// across workgroups; the in-group part lives in the main kernel.
//
// Each thread owns four consecutive outputs (the host keeps every slice a multiple of four
// elements long, so the 16-byte loads stay inside their slice) and reads the first eight slices
// at once: a slice index past the last one re-reads the last slice and is not added, which keeps
// the loads free of branches.  All loads of the requantise inputs go through buffer descriptors
// (an absent input has an empty range and reads as zero) and come before the first store.
template <typename E>
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const ReduceArgs a)
{
    typedef E v4e __attribute__((ext_vector_type(4)));
    const int total = (int)a.total;                  // < 2^29: the output stays below 2 GiB
    const int i = (int)(blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= total) return;
    const E *p = reinterpret_cast<const E *>(a.partials) + i;
    const int last = a.nsplit - 1;
    v4e head[8];
#pragma unroll
    for (int z = 0; z < 8; ++z)
        head[z] = *reinterpret_cast<const v4e *>(p + (long)(z < last ? z : last) * a.split_stride);
    v4e sum = head[0];
#pragma unroll
    for (int z = 1; z < 8; ++z) {                    // fixed order z = 1, 2, 3, ...: deterministic for fp32
        const v4e zero = {0, 0, 0, 0};
        sum += (z <= last) ? head[z] : zero;
    }
    for (int z = 8; z <= last; ++z) sum += *reinterpret_cast<const v4e *>(p + (long)z * a.split_stride);

    const bool full = i + 3 < total;
    if (a.out) {
        E *o = reinterpret_cast<E *>(a.out) + i;
        if (full) {
            *reinterpret_cast<v4e *>(o) = sum;       // (a global 16-byte store needs 4-byte alignment only)
        } else {
#pragma unroll
            for (int e = 0; e < 3; ++e)
                if (i + e < total) o[e] = sum[e];
        }
    }
    if (a.epi != EPI_REQUANT) return;

    const __amdgpu_buffer_rsrc_t rsS = make_rsrc(a.scale, UNIT_OOB);
    const __amdgpu_buffer_rsrc_t rsB = make_rsrc(a.bias, a.bias ? UNIT_OOB : 0u);
    const __amdgpu_buffer_rsrc_t rsR = make_rsrc(a.residual, a.residual ? UNIT_OOB : 0u);
    const __amdgpu_buffer_rsrc_t rsP = make_rsrc(a.res_packed, a.res_packed ? UNIT_OOB : 0u);
    int t[4];  float sc[4];  unsigned pk[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int idx = (i + e < total) ? i + e : i;              // a lane past the end repeats element i
        const int nk = div_any(idx, a.PQ);
        const int px = idx - nk * a.PQ;
        const int n = div_any(nk, a.K);
        const int k = nk - n * a.K;
        pk[e] = (unsigned)((n * a.PQ + px) * a.packed_ld + k);
        unsigned u = (unsigned)(int)sum[e];
        u += __builtin_amdgcn_raw_buffer_load_b32(rsB, (unsigned)k * 4u, 0, 0);
        u += __builtin_amdgcn_raw_buffer_load_b32(rsR, (unsigned)idx * 4u, 0, 0);
        const int r8 = (int)(int8_t)__builtin_amdgcn_raw_buffer_load_b8(rsP, pk[e], 0, 0);
        u += (unsigned)(r8 * a.res_mult);
        t[e] = (int)u;
        sc[e] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsS, (unsigned)k * 4u, 0, 0));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (i + e >= total) break;
        const int v = requant_elem(t[e], sc[e], a.relu);
        if (a.out_i8) a.out_i8[i + e] = (int8_t)v;
        if (a.out_packed) a.out_packed[pk[e]] = (int8_t)v;
    }
}

// zero the padding channels [K, packed_ld) of a packed int8 output
__global__ void zero_pad_channels_kernel(int8_t *yp, int K, int ld, long pixels)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    int npad = ld - K;
    if (i >= pixels * npad) return;
    yp[(i / npad) * ld + K + i % npad] = 0;
}

hipError_t launch_splitk_reduce(const ReduceArgs &a, hipStream_t st)
{
    // the requantise epilogue derives the channel from the element index
    if (a.total <= 0 || a.nsplit < 1 || (a.epi == EPI_REQUANT && (a.K <= 0 || a.PQ <= 0))) return hipErrorInvalidValue;
    dim3 grid((unsigned)((a.total + 1023) / 1024)), block(256);
    if (a.dtype == DT_I8) hipLaunchKernelGGL(splitk_reduce_kernel<int>, grid, block, 0, st, a);
    else                  hipLaunchKernelGGL(splitk_reduce_kernel<float>, grid, block, 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.epi == EPI_REQUANT && a.out_packed && a.packed_ld > a.K) {
        long pixels = a.total / a.K;
        long cnt = pixels * (a.packed_ld - a.K);
        hipLaunchKernelGGL(zero_pad_channels_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st,
                           a.out_packed, a.K, a.packed_ld, pixels);
        e = hipGetLastError();
    }
    return e;
}

// ------------------------------------------------------------------ unsigned-operand correction
// out[r] = 128 * (sum of the signed bytes of row r); rows are `ld` bytes apart, 16-byte
// aligned and `chunks` 16-byte chunks long.  One wave per row.
__global__ void __launch_bounds__(256)
rowsum128_i8_kernel(const uint8_t *__restrict__ m, long ld, int rows, int chunks, int32_t *__restrict__ out)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= rows) return;
    const v4i *p = reinterpret_cast<const v4i *>(m + (long)row * ld);
    int sum = 0;
    for (int c = lane; c < chunks; c += 64) {
        v4i v = p[c];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            int w = v[d];
            sum += (int)(int8_t)(w & 0xff) + (int)(int8_t)((w >> 8) & 0xff) +
                   (int)(int8_t)((w >> 16) & 0xff) + (w >> 24);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) out[row] = sum * 128;
}

hipError_t launch_rowsum128_i8(const void *m, long ld, int rows, int chunks, int32_t *out, hipStream_t st)
{
    hipLaunchKernelGGL(rowsum128_i8_kernel, dim3((rows + 3) / 4), dim3(256), 0, st,
                       static_cast<const uint8_t *>(m), ld, rows, chunks, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ matmul with very few rows
// C[r][col] = sum_k A[r][k] * B[col][k] for a handful of rows (the fully connected layer of batch-1 inference: the paper's
// matmul with one row, Section II-A).  The matrix units would run 15/16 empty and, worse, a 16 x 64 tile leaves
// only n / 64 workgroups to stream B, the one operand of any size.  Here one wave owns one output column: it reads
// that column's reduction row of B once, 16 bytes per lane and load, multiplies each chunk with the same chunk of
// every row of A by the dot-product instructions of the vector ALU (v_dot4_i32_i8: four byte products added into an
// int32, exact; v_dot2_f32_f16: two half products added into an fp32) and adds the lanes' sums with a butterfly.
// n / 4 workgroups keep every compute unit streaming.  Rows of both operands start 16-byte aligned and are
// `kchunks` 16-byte chunks long (the caller pads otherwise).  MR = compiled number of rows (rows past m repeat row 0
// and are not stored).
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

template <int DT, int MR>
__global__ void __launch_bounds__(256)
gemv_kernel(const uint8_t *__restrict__ A, long lda, const uint8_t *__restrict__ B, long ldb,
            int m, int n, int kchunks, void *__restrict__ C, long ldc)
{
    typedef typename Mma<DT, 32>::elem_t elem_t;
    const int col = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (col >= n) return;
    const v4i *b = reinterpret_cast<const v4i *>(B + (long)col * ldb);
    const v4i *a[MR];
#pragma unroll
    for (int r = 0; r < MR; ++r) a[r] = reinterpret_cast<const v4i *>(A + (long)(r < m ? r : 0) * lda);
    elem_t acc[MR];
#pragma unroll
    for (int r = 0; r < MR; ++r) acc[r] = 0;
    auto mac = [&](const v4i &bv, const v4i &av, elem_t &c) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int ai = av[d], bi = bv[d];       // (values, not vector-element lvalues: those do not bit_cast element-wise)
            if constexpr (DT == DT_I8) {
                c = __builtin_amdgcn_sdot4(ai, bi, c, false);
            } else {
                c = __builtin_amdgcn_fdot2(__builtin_bit_cast(v2h, ai), __builtin_bit_cast(v2h, bi), c, false);
            }
        }
    };
    // two chunks per lane and trip: all loads of a trip are issued before the first multiply
    int c = lane;
    for (; c + 64 < kchunks; c += 128) {
        const v4i b0 = b[c], b1 = b[c + 64];
        v4i a0[MR], a1[MR];
#pragma unroll
        for (int r = 0; r < MR; ++r) { a0[r] = a[r][c];  a1[r] = a[r][c + 64]; }
#pragma unroll
        for (int r = 0; r < MR; ++r) { mac(b0, a0[r], acc[r]);  mac(b1, a1[r], acc[r]); }
    }
    if (c < kchunks) {
        const v4i b0 = b[c];
#pragma unroll
        for (int r = 0; r < MR; ++r) mac(b0, a[r][c], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < MR; ++r) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc[r] += __shfl_xor(acc[r], off, 64);
    }
    if (lane == 0) {
        elem_t *out = static_cast<elem_t *>(C);
#pragma unroll
        for (int r = 0; r < MR; ++r)
            if (r < m) out[(long)r * ldc + col] = acc[r];
    }
}

template <int DT>
static hipError_t launch_gemv_dt(const void *A, long lda, const void *B, long ldb, int m, int n, int kchunks,
                                 void *C, long ldc, hipStream_t st)
{
    const dim3 grid((n + 3) / 4), block(256);
    const uint8_t *a = static_cast<const uint8_t *>(A), *b = static_cast<const uint8_t *>(B);
    if (m == 1)      hipLaunchKernelGGL((gemv_kernel<DT, 1>), grid, block, 0, st, a, lda, b, ldb, m, n, kchunks, C, ldc);
    else if (m == 2) hipLaunchKernelGGL((gemv_kernel<DT, 2>), grid, block, 0, st, a, lda, b, ldb, m, n, kchunks, C, ldc);
    else if (m <= 4) hipLaunchKernelGGL((gemv_kernel<DT, 4>), grid, block, 0, st, a, lda, b, ldb, m, n, kchunks, C, ldc);
    else             hipLaunchKernelGGL((gemv_kernel<DT, 8>), grid, block, 0, st, a, lda, b, ldb, m, n, kchunks, C, ldc);
    return hipGetLastError();
}

// dtype: DT_I8 or DT_F16; m <= 8 (the API uses it up to GEMV_MAX_ROWS); lda, ldb in bytes
hipError_t launch_gemv(int dtype, const void *A, long lda, const void *B, long ldb, int m, int n, int kchunks,
                       void *C, long ldc, hipStream_t st)
{
    if (m < 1 || m > 8) return hipErrorInvalidValue;
    if (dtype == DT_I8) return launch_gemv_dt<DT_I8>(A, lda, B, ldb, m, n, kchunks, C, ldc, st);
    if (dtype == DT_F16) return launch_gemv_dt<DT_F16>(A, lda, B, ldb, m, n, kchunks, C, ldc, st);
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------ int8 network glue
// max-pool on packed int8: one thread per (n, p, q, 16-channel chunk).  With a compile-time
// window (WIN > 0) all window loads are issued at once through a buffer descriptor (taps in the
// padding get an out-of-range offset and are replaced by -128 afterwards); WIN == 0 walks a
// window of any size.
template <int WIN>
__global__ void __launch_bounds__(256)
maxpool_packed_i8_kernel(const int8_t *__restrict__ x, int8_t *__restrict__ y,
                         int cp, int H, int W, int P, int Q,
                         int window, int stride, int pad, int total, unsigned x_bytes)
{
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i >= total) return;
    const int chunks = cp / 16;
    int t = div_any(i, chunks);
    const int cc = i - t * chunks;
    const int t2 = div_any(t, Q);
    const int q = t - t2 * Q;
    const int n = div_any(t2, P);
    const int p = t2 - n * P;
    int best[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) best[e] = -128;
    auto take = [&](const v4i &raw) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int b = (int)(int8_t)((unsigned)raw[e >> 2] >> (8 * (e & 3)));
            best[e] = (b > best[e]) ? b : best[e];
        }
    };
    if (WIN > 0) {
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(x, x_bytes);
        v4i raw[WIN > 0 ? WIN * WIN : 1];
#pragma unroll
        for (int r = 0; r < WIN; ++r)
#pragma unroll
            for (int s2 = 0; s2 < WIN; ++s2) {
                const int h = p * stride + r - pad, w = q * stride + s2 - pad;
                const bool ok = (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
                v4i v = buf_load16(rs, ok ? (unsigned)(((n * H + h) * W + w) * cp + cc * 16) : UNIT_OOB);
                const v4i lowest = {(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
                raw[r * WIN + s2] = ok ? v : lowest;
            }
#pragma unroll
        for (int k = 0; k < WIN * WIN; ++k) take(raw[k]);
    } else {
        for (int r = 0; r < window; ++r) {
            const int h = p * stride + r - pad;
            if (h < 0 || h >= H) continue;
            for (int s2 = 0; s2 < window; ++s2) {
                const int w = q * stride + s2 - pad;
                if (w < 0 || w >= W) continue;
                take(*reinterpret_cast<const v4i *>(x + ((long)(n * H + h) * W + w) * cp + cc * 16));
            }
        }
    }
    __attribute__((aligned(16))) int8_t outv[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) outv[e] = (int8_t)best[e];
    *reinterpret_cast<v4i *>(y + ((long)(n * P + p) * Q + q) * cp + cc * 16) = *reinterpret_cast<const v4i *>(outv);
}

hipError_t launch_maxpool_packed_i8(int n, int cp, int h, int w, int window, int stride, int pad,
                                    int p, int q, const void *x, void *y, hipStream_t st)
{
    const long total = (long)n * p * q * (cp / 16);
    const long x_bytes = (long)n * h * w * cp;
    if (total >= (1L << 31) || x_bytes >= (1L << 31)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (window == 3)
        hipLaunchKernelGGL(maxpool_packed_i8_kernel<3>, grid, block, 0, st, (const int8_t *)x, (int8_t *)y, cp, h, w,
                           p, q, window, stride, pad, (int)total, (unsigned)x_bytes);
    else if (window == 2)
        hipLaunchKernelGGL(maxpool_packed_i8_kernel<2>, grid, block, 0, st, (const int8_t *)x, (int8_t *)y, cp, h, w,
                           p, q, window, stride, pad, (int)total, (unsigned)x_bytes);
    else
        hipLaunchKernelGGL(maxpool_packed_i8_kernel<0>, grid, block, 0, st, (const int8_t *)x, (int8_t *)y, cp, h, w,
                           p, q, window, stride, pad, (int)total, (unsigned)x_bytes);
    return hipGetLastError();
}

// global average pool: integer sum then requantise.  One workgroup per (image, 64 channels):
// thread = (pixel slice, channel quad); every thread sums its slice of the pixels with 32-bit
// loads of four channels, the 16 slices are added through LDS, and 64 threads requantise.
__global__ void __launch_bounds__(256)
avgpool_packed_i8_kernel(const int8_t *__restrict__ x, const float *__restrict__ scale,
                         int8_t *__restrict__ y, int C, int cp, int HW, int groups)
{
    __shared__ int part[16][64];
    const int quad = threadIdx.x & 15, slice = threadIdx.x >> 4;
    const int grp = blockIdx.x % groups;
    const long n = blockIdx.x / groups;
    const int c0 = (grp * 16 + quad) * 4;               // first of this thread's four channels
    int s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    if (c0 < cp) {
        const int8_t *px = x + (n * HW + slice) * (long)cp + c0;
        for (int i = slice; i < HW; i += 16, px += 16L * cp) {
            const unsigned v = *reinterpret_cast<const unsigned *>(px);
            s0 += (int)(int8_t)v;  s1 += (int)(int8_t)(v >> 8);
            s2 += (int)(int8_t)(v >> 16);  s3 += (int)(int8_t)(v >> 24);
        }
    }
    part[slice][quad * 4 + 0] = s0;  part[slice][quad * 4 + 1] = s1;
    part[slice][quad * 4 + 2] = s2;  part[slice][quad * 4 + 3] = s3;
    __syncthreads();
    if (threadIdx.x < 64) {
        const int c = grp * 64 + threadIdx.x;
        if (c < cp) {
            int sum = 0;
#pragma unroll
            for (int t = 0; t < 16; ++t) sum += part[t][threadIdx.x];
            y[n * cp + c] = c < C ? (int8_t)requant_elem(sum, scale[c], 0) : (int8_t)0;
        }
    }
}

hipError_t launch_avgpool_packed_i8(int n, int c, int cp, int hw, const void *x, const float *scale,
                                    int8_t *y, hipStream_t st)
{
    const int groups = (cp + 63) / 64;
    hipLaunchKernelGGL(avgpool_packed_i8_kernel, dim3((unsigned)((long)n * groups)), dim3(256), 0, st,
                       (const int8_t *)x, scale, y, c, cp, hw, groups);
    return hipGetLastError();
}

__global__ void widen_residual_i8_kernel(const int8_t *__restrict__ x, int32_t *__restrict__ res,
                                         int C, int cp, int HW, int mult, long total)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;   // NCHW index
    if (i >= total) return;
    int px = i % HW;
    long nc = i / HW;
    int c = nc % C;
    long n = nc / C;
    res[i] = (int)x[(n * HW + px) * cp + c] * mult;
}

hipError_t launch_widen_residual_i8(int n, int c, int cp, int hw, const void *x, int mult,
                                    int32_t *res, hipStream_t st)
{
    long total = (long)n * c * hw;
    hipLaunchKernelGGL(widen_residual_i8_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const int8_t *)x, res, c, cp, hw, mult, total);
    return hipGetLastError();
}

}  // namespace unit
