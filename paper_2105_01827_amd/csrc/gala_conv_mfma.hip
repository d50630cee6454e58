// The convolution's ScMult/Add step on the matrix cores.
//
// For one coefficient index i the step is a dense product  S_i[m][c] = sum_k W_i[m][k] * X_i[k][c]  of 60-bit
// residues (m: output block x kernel order, k: input ciphertext x tap, c: input x polynomial), accumulated
// exactly and reduced mod q once at the end.  It is mapped on the int8 MFMA units by writing every residue in
// eight balanced base-256 digits d_0..d_7 in [-128,127] (x = sum d_u 256^u): then
//     S = sum_{s=0..14} 256^s * D_s,   D_s[m][c] = sum_{u+v=s} sum_k W_u[m][k] * X_v[k][c]
// and every D_s is an int8 x int8 -> int32 matrix product (|D_s| <= 8 * 192 * 2^14 < 2^31 and S < 192 * 2^120 < 2^128
// for the at most 192 terms summed between two reductions mod q, given q < 2^60: exact).
// One v_mfma_i32_16x16x64_i8 multiplies a 16x64 by a 64x16 digit tile; the 64 (u,v) digit pairs of a tile feed
// 15 accumulators of four registers each.  The recombination of the 15 diagonals, the reduction mod q and the
// transposition back to coefficient-major order run on the vector ALU in the same kernel.
//
// Operand images ("digit planes") are made of 16-byte chunks: lane l of the MFMA holds row/column l%16 of a
// tile and the 16 terms k = 64*kblock + 16*(l/16) + j of one digit.
//   row operand (encoded kernels):     [i][tile][kblock][digit][lane]   one digit plane of a tile is 1 KiB
//   column operand (rotated inputs):   [tile][kblock][lane][i][digit]   the 8 digits of a coefficient are 128 B
// The column layout lets the kernel that produces the rotated inputs write it with the coefficient index
// running across the lanes.  Chunks whose 16 terms all lie beyond the last term are never read.
#include <hip/hip_runtime.h>

#include "gala_internal.h"

namespace gala {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// term blocks of 64 between two reductions of the running sums (conv_mfma_kernel); q < 2^60 is required
constexpr int kFoldBlocks = 3;

// balanced base-256 digits of x < 2^61, one per byte: the bytes of x + 0x80..80 are the digits plus 128
__device__ __forceinline__ u64 balanced_digits(u64 x) {
    const u64 k = 0x8080808080808080ull;
    return (x + k) ^ k;
}

// the 16 bytes of digit `limb` of 16 balanced-digit words
__device__ __forceinline__ v4i digit_chunk(const u64 (&d)[16], int limb) {
    v4i c;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        u32 wd = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) wd |= (u32)((d[4 * t + b] >> (8 * limb)) & 0xff) << (8 * b);
        c[t] = (int)wd;
    }
    return c;
}

// Builds the digit-plane image of 16 rows x 16 terms x 16 coefficients per workgroup.  Phase 1 reads the
// source with the coefficient index fastest (128-byte segments); phase 2 writes with the index fastest that
// is contiguous in the destination layout.  mode 0: source is the encoded
// kernels [row][e][i]; mode 1: the tap-rotated inputs [input][e][polynomial][i] with row = 2*input + polynomial.
__global__ __launch_bounds__(256) void limb_pack_kernel(const u64 *src, int mode, int rows, int nterm, int n, int tiles,
                                                        int kblocks, v4i *dst) {
    __shared__ u64 stage[16 * 16 * 17];   // [row][term][coefficient], coefficient dimension padded
    const int i0 = blockIdx.x * 16, tile = blockIdx.y, kb = blockIdx.z >> 2, g = blockIdx.z & 3;
    {
        const int il = threadIdx.x & 15, rl = threadIdx.x >> 4, row = tile * 16 + rl;
        const size_t row_off = mode == 0 ? (size_t)row * nterm * n : ((size_t)(row >> 1) * nterm * 2 + (row & 1)) * n;
        const size_t e_stride = mode == 0 ? (size_t)n : 2 * (size_t)n;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int e = kb * 64 + g * 16 + j;
            const u64 x = (row < rows && e < nterm && i0 + il < n) ? src[row_off + (size_t)e * e_stride + i0 + il] : 0;
            stage[(rl * 16 + j) * 17 + il] = balanced_digits(x);
        }
    }
    __syncthreads();
    // phase 2: mode 0 runs the row across the threads, mode 1 the coefficient
    const int rl = mode == 0 ? threadIdx.x & 15 : threadIdx.x >> 4, il = mode == 0 ? threadIdx.x >> 4 : threadIdx.x & 15;
    const bool live = i0 + il < n;
    u64 d[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) d[j] = stage[(rl * 16 + j) * 17 + il];
    const size_t lane = (size_t)(g * 16 + rl);
    if (mode == 0) {
        if (!live) return;
        // 16 threads (the rows of a tile) write 256 contiguous bytes per digit
        const size_t base = ((((size_t)(i0 + il) * tiles + tile) * kblocks + kb) * 8) * 64 + lane;
#pragma unroll
        for (int limb = 0; limb < 8; ++limb) dst[base + (size_t)limb * 64] = digit_chunk(d, limb);
        return;
    }
    // mode 1: a row's 16 coefficients x 8 digits are 2 KiB contiguous in the image, but a thread owns the 128
    // bytes of one coefficient: the chunks change owner in LDS so that the 16 threads of a row write 256
    // contiguous bytes per instruction instead of 16 bytes in each of 16 lines
    __syncthreads();                                   // everybody has read its digits out of `stage`
    v4i *tr = reinterpret_cast<v4i *>(stage);          // [row][coefficient][digit], 32 KiB
#pragma unroll
    for (int limb = 0; limb < 8; ++limb) tr[(rl * 16 + il) * 8 + limb] = digit_chunk(d, limb);
    __syncthreads();
    const size_t base = ((((size_t)tile * kblocks + kb) * 64 + lane) * n + i0) * 8;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int c = k * 16 + il;                     // chunk c of the row: coefficient c / 8, digit c % 8
        if (i0 + (c >> 3) < n) dst[base + c] = tr[rl * 128 + c];
    }
}

// sum_s 256^s * c[s] for 15 signed 32-bit diagonals, as an unsigned 128-bit value (the true sum is non-negative).
// Four diagonals at a time fit a signed 64-bit word (|e| < 2^56); the four words, 32 bits apart, are then added
// with 32-bit carries.
__device__ __forceinline__ u128 recombine(const int (&c)[15]) {
    // the multipliers are hidden from the optimiser so that each term is one 32x32+64 multiply-add instead of a
    // sign extension, a 64-bit shift and a 64-bit addition
    int m8 = 256, m16 = 65536, m24 = 16777216;
    asm volatile("" : "+s"(m8), "+s"(m16), "+s"(m24));
    i64 e[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        e[j] = (i64)c[4 * j] + (i64)c[4 * j + 1] * m8 + (i64)c[4 * j + 2] * m16;
        if (j < 3) e[j] += (i64)c[4 * j + 3] * m24;
    }
    i64 t = e[0];
    const u64 w0 = (uint32_t)t;
    t = (t >> 32) + e[1];
    const u64 w1 = (uint32_t)t;
    t = (t >> 32) + e[2];
    const u64 w2 = (uint32_t)t;
    t = (t >> 32) + e[3];
    const u64 w3 = (uint32_t)t;
    return ((u128)(w2 | (w3 << 32)) << 64) | (w0 | (w1 << 32));
}

// One workgroup = one coefficient, WAVES row tiles (one per wavefront) and 2 column tiles.  The column
// operand (rotated inputs) of a term block is staged once in LDS and read by all wavefronts; every wavefront
// streams its own row operand (encoded kernels) from memory, so each operand byte is fetched once per
// workgroup.  Loads of the next term block are issued before the MFMAs of the current one.
// Output: tmp[i][row][column] (rows and columns padded to tiles), transposed afterwards; or, BLK8, in blocks of
// eight coefficients tmp[i/8][row][column][i%8], which the n = 2048 Perm kernel reads as they are (a thread's eight
// consecutive coefficients of c0 and of c1 are the two halves of one 128-byte line).
template <int WAVES, bool BLK8, bool FOLD>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void conv_mfma_kernel(const v4i *wl, const v4i *xl, u64 *tmp, int mtiles,
                                                               int ntiles, int kblocks, int nblk16, int n, Modulus mod) {
    constexpr int NT = 64 * WAVES, BLOADS = 1024 / NT;
    __shared__ v4i bsm[2][2][8][64];     // [buffer][column tile][digit][lane], 32 KiB
    // the wavefront's number is the same in all its lanes: kept in a scalar register, with everything derived from it
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // BLK8: eight consecutive coefficients are handled by workgroups 8 apart, which run on the same XCD
    const size_t i = BLK8 ? (size_t)(blockIdx.x & 7) * (n >> 3) + (blockIdx.x >> 3) : (size_t)blockIdx.x;
    const int mt = blockIdx.y * WAVES + wave, nt0 = blockIdx.z * 2;
    const bool live = mt < mtiles;
    const int mtc = live ? mt : mtiles - 1;
    const v4i zero = v4i{0, 0, 0, 0};
    // cooperative load of the column operand: 2 tiles x 64 lanes x 8 digits chunks, BLOADS per thread, with the
    // digit fastest (128 contiguous bytes per lane); chunks beyond the last term block are zero without a load
    auto b_load = [&](int kb, int r) -> v4i {
        const int c = threadIdx.x + NT * r, nl = c >> 9, ln = (c >> 3) & 63, dg = c & 7;
        const int nt = min(nt0 + nl, ntiles - 1);
        if (kb * 4 + (ln >> 4) >= nblk16) return zero;
        return xl[((((size_t)nt * kblocks + kb) * 64 + ln) * n + i) * 8 + dg];
    };
    auto b_slot = [&](int r) { const int c = threadIdx.x + NT * r; return (c >> 9) * 512 + (c & 7) * 64 + ((c >> 3) & 63); };
    auto a_load = [&](int kb, v4i (&dst)[8]) {
        const v4i *a = wl + (((i * mtiles + mtc) * kblocks + kb) * 8) * 64 + lane;
        const bool on = kb * 4 + (lane >> 4) < nblk16;
#pragma unroll
        for (int u = 0; u < 8; ++u) dst[u] = on ? a[(size_t)u * 64] : zero;
    };
    v4i s[2][15];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int k = 0; k < 15; ++k) s[t][k] = v4i{0, 0, 0, 0};
    v4i av[8], an[8], bstage[BLOADS];
#pragma unroll
    for (int r = 0; r < BLOADS; ++r) bstage[r] = b_load(0, r);
    a_load(0, av);
    for (int kb = 0; kb < kblocks; ++kb) {
        v4i *flat = &bsm[kb & 1][0][0][0];
#pragma unroll
        for (int r = 0; r < BLOADS; ++r) flat[b_slot(r)] = bstage[r];
        __syncthreads();     // the other buffer was last read two barriers ago
        const int nxt = min(kb + 1, kblocks - 1);
#pragma unroll
        for (int r = 0; r < BLOADS; ++r) bstage[r] = b_load(nxt, r);
        a_load(nxt, an);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            v4i bv[8];
#pragma unroll
            for (int v = 0; v < 8; ++v) bv[v] = bsm[kb & 1][t][v][lane];
            // column-major over the digit pairs: the same accumulator comes back only every seventh instruction
#pragma unroll
            for (int v = 0; v < 8; ++v)
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    s[t][u + v] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[u], bv[v], s[t][u + v], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) av[u] = an[u];
        // The exact sum of K products of residues below 2^60 needs K * 2^120 < 2^128, and an int32 diagonal
        // 8 * K * 2^14 < 2^31: after every kFoldBlocks term blocks (192 terms) the sums so far are reduced mod q
        // and put back as three small non-negative diagonals (24 + 24 + 12 bits at 256^0, 256^3, 256^6), so sums
        // of any length stay exact.  Layers of at most 192 terms run the instantiation without this branch (FOLD =
        // false: the branch costs three spilled registers that the main loop reloads).
        if (FOLD && kb % kFoldBlocks == kFoldBlocks - 1 && kb + 1 < kblocks) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    int c[15];
#pragma unroll
                    for (int k = 0; k < 15; ++k) c[k] = s[t][k][r];
                    const u64 val = reduce128(recombine(c), mod);
#pragma unroll
                    for (int k = 0; k < 15; ++k) s[t][k][r] = 0;
                    s[t][0][r] = (int)(val & 0xffffff);
                    s[t][3][r] = (int)((val >> 24) & 0xffffff);
                    s[t][6][r] = (int)(val >> 48);
                }
        }
    }
    if (!live) return;
    // lane holds rows 4*(lane/16) + r, column lane%16 of each 16x16 output tile
    const size_t rowsP = (size_t)mtiles * 16, colsP = (size_t)ntiles * 16;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (nt0 + t >= ntiles) break;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int c[15];
#pragma unroll
            for (int k = 0; k < 15; ++k) c[k] = s[t][k][r];
            const u64 val = reduce128(recombine(c), mod);
            const int m = mt * 16 + 4 * (lane >> 4) + r, col = (nt0 + t) * 16 + (lane & 15);
            if (BLK8) tmp[(((i >> 3) * rowsP + m) * colsP + col) * 8 + (i & 7)] = val;
            else tmp[(i * rowsP + m) * colsP + col] = val;
        }
    }
}

// acc[input][row][polynomial][i] = tmp[i][row][2*input + polynomial]: a tiled transpose through LDS
__global__ __launch_bounds__(256) void conv_untranspose_kernel(const u64 *tmp, u64 *acc, int rowsP, int colsP, int groups,
                                                               int cols, int n) {
    __shared__ u64 tile[32][33];
    const int i0 = blockIdx.x * 32, r0 = blockIdx.y * 32;       // r = row * colsP + column, flattened
    const size_t flat = (size_t)rowsP * colsP;
    for (int k = threadIdx.x; k < 32 * 32; k += 256) {
        const int di = k >> 5, dr = k & 31;
        if (i0 + di < n && (size_t)(r0 + dr) < flat) tile[di][dr] = tmp[(size_t)(i0 + di) * flat + r0 + dr];
    }
    __syncthreads();
    for (int k = threadIdx.x; k < 32 * 32; k += 256) {
        const int dr = k >> 5, di = k & 31;
        const int r = r0 + dr, row = r / colsP, col = r % colsP;
        if (i0 + di < n && row < groups && col < cols)
            acc[(((size_t)(col >> 1) * groups + row) * 2 + (col & 1)) * n + i0 + di] = tile[di][dr];
    }
}

}  // namespace

void conv_mfma_geometry(int groups, int cols, int nterm, int *mtiles, int *ntiles, int *kblocks) {
    *mtiles = (groups + 15) / 16;
    *ntiles = (cols + 15) / 16;
    *kblocks = (nterm + 63) / 64;
}
size_t conv_mfma_image_bytes(int n, int tiles, int kblocks) {
    return (size_t)n * tiles * kblocks * 8 * 64 * 16;
}
size_t conv_mfma_tmp_bytes(int n, int mtiles, int ntiles) { return (size_t)n * mtiles * 16 * ntiles * 16 * sizeof(u64); }
// mode 0: encoded kernels (rows = groups), mode 1: rotated inputs (rows = 2*batch columns)
int launch_limb_pack(const gala_ctx *c, void *stream, const u64 *src, int mode, int rows, int nterm, u64 *dst) {
    int tiles, unused, kblocks;
    conv_mfma_geometry(rows, rows, nterm, &tiles, &unused, &kblocks);
    const dim3 grid((unsigned)((c->n + 15) / 16), (unsigned)tiles, (unsigned)(kblocks * 4));
    hipLaunchKernelGGL(limb_pack_kernel, grid, dim3(256), 0, (hipStream_t)stream, src, mode, rows, nterm, c->n, tiles,
                       kblocks, reinterpret_cast<v4i *>(dst));
    return (int)hipGetLastError();
}
int launch_conv_mfma(const gala_ctx *c, void *stream, const u64 *wl, const u64 *xl, int batch, int groups, int nterm,
                     u64 *tmp, bool blocks_of_eight) {
    int mtiles, ntiles, kblocks;
    conv_mfma_geometry(groups, 2 * batch, nterm, &mtiles, &ntiles, &kblocks);
    constexpr int WAVES = 4;
    const dim3 grid((unsigned)c->n, (unsigned)((mtiles + WAVES - 1) / WAVES), (unsigned)((ntiles + 1) / 2));
    const bool fold = kblocks > kFoldBlocks;
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(64 * WAVES), 0, (hipStream_t)stream, reinterpret_cast<const v4i *>(wl),
                           reinterpret_cast<const v4i *>(xl), tmp, mtiles, ntiles, kblocks, (nterm + 15) / 16, c->n,
                           c->dev_q.mod);
    };
    if (blocks_of_eight) fold ? go(conv_mfma_kernel<WAVES, true, true>) : go(conv_mfma_kernel<WAVES, true, false>);
    else fold ? go(conv_mfma_kernel<WAVES, false, true>) : go(conv_mfma_kernel<WAVES, false, false>);
    return (int)hipGetLastError();
}
int launch_conv_untranspose(const gala_ctx *c, void *stream, const u64 *tmp, int batch, int groups, u64 *acc) {
    int mtiles, ntiles, kblocks;
    const int cols = 2 * batch;
    conv_mfma_geometry(groups, cols, 1, &mtiles, &ntiles, &kblocks);
    const int rowsP = mtiles * 16, colsP = ntiles * 16;
    const dim3 tgrid((unsigned)((c->n + 31) / 32), (unsigned)((rowsP * colsP + 31) / 32));
    hipLaunchKernelGGL(conv_untranspose_kernel, tgrid, dim3(256), 0, (hipStream_t)stream, tmp, acc, rowsP, colsP, groups,
                       cols, c->n);
    return (int)hipGetLastError();
}

}  // namespace gala
