// Decoder projections y[m][n] = sum_k x[m][k] W[n][k] on gfx950.
//
// The kernels, chosen by model dtype and row count M (M = batch * n_new of a verify step):
//   gemm_f32_kernel          fp32 weights, plain ALU dot products, one wavefront per output
//                            column (the tiny fp32 chain; fp32 1e-4 parity, not speed).
//   gemm_bf16_skinny_kernel  M <= 16, weights as the caller stores them (row-major).  HBM-bound weight
//                            streaming: W rows go straight from global memory into MFMA A-operand registers
//                            with 16-byte loads (no LDS), the few activation rows are the B operand, K is
//                            split over the four wavefronts of a block and over blocks.
//   gemm_bf16_unit_kernel    M <= 16 on weights repacked by gemm_pack_kernel: the same MFMA tiling, but every
//                            16 KB unit (64 rows x 128 k) is stored in exactly the order the lanes load it,
//                            units of a GEMM are contiguous, and the grid is persistent: each block streams
//                            an equal, contiguous range of units (stream-K), its four wavefronts on the four
//                            K quarters of every unit, and writes one partial per tile it touches.
//                            With RESID (the down projection) the block that arrives last at a tile adds the
//                            tile's partials and runs the residual epilogue below.
//   gemm_bf16_column_kernel  M <= 16, the O projection (it writes the residual stream and is short along K): one
//                            block per 16 output columns over the whole K range; the residual add, the
//                            gain-scaled copy and the RMSNorm statistics happen in its epilogue.
//   gemm_w4_unit_kernel      M <= 16, 4-bit weight-only quantised projections (groups of 128 along K): the unit
//                            kernel's stream-K over quads of four K steps, the codes multiplied as exact fp16
//                            integers against fp16-rounded activations, scale and zero point applied per group in
//                            fp32; one partial slot per block and tile, or (O, down) the residual epilogue run by
//                            the block that arrives last.
//   gemm_f16_tiled_kernel    M > 16.  (128 or 256) x (128, 192, 256) x 64 LDS-staged tiles, 32x32x16 fp16 MFMA
//                            (weights convert to fp16 exactly, activations are rounded to fp16).
// Activations are fp32 in memory in every case (the tiled kernel reads an fp16 copy its producers leave beside
// them).  The M <= 16 bf16 kernels feed each activation to the matrix cores as a pair of bf16 values hi + lo (two
// MFMAs against the same weight operand): with plain bf16 activations the logits of the 7B-shaped random-init
// models are 3e-2 off the fp64 result, above the 2e-2 bar; the weights, which are what streams from HBM, stay bf16.
// Every kernel but the ones with the residual epilogue writes its result as split-K partials [splitk][M][N]
// (splitk >= 1); the consumer (the fused row-wise kernels, the attention kernel's operand build, or
// gemm_splitk_reduce_kernel for the logits) adds them in split order, so results are bit-reproducible.
#include <type_traits>
#include "common.h"
#include "kernels.h"
#include "prof.h"
#include "../../include/psd.h"

namespace psd {
namespace {

// source row of activation row m: rows may be a strided subset (the last rows of each sequence)
__host__ __device__ __forceinline__ size_t x_row(const GemmArgs &g, int m) {
    return (size_t)(m / g.x_rows_per_group) * g.x_group_stride + g.x_group_offset + (m % g.x_rows_per_group);
}

// ------------------------------------------------------------------------------ fp32
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + wave;
    if (n >= g.N) return;
    int seg = 0, nl = n;
    while (seg < g.nseg - 1 && nl >= g.n[seg]) { nl -= g.n[seg]; ++seg; }
    const float *wrow = (const float *)g.w[seg] + (size_t)nl * g.K;
    const float *x = (const float *)g.x;
    for (int m0 = 0; m0 < g.M; m0 += 8) {
        float acc[8];
#pragma unroll
        for (int mm = 0; mm < 8; ++mm) acc[mm] = 0.f;
        for (int k = lane; k < g.K; k += 64) {
            const float w = wrow[k];
#pragma unroll
            for (int mm = 0; mm < 8; ++mm)
                if (m0 + mm < g.M) acc[mm] += w * x[x_row(g, m0 + mm) * g.K + k];
        }
#pragma unroll
        for (int mm = 0; mm < 8; ++mm) acc[mm] = wave_sum(acc[mm]);
        if (lane == 0) {
#pragma unroll
            for (int mm = 0; mm < 8; ++mm)
                if (m0 + mm < g.M) {
                    g.partial[(size_t)(m0 + mm) * g.N + n] = acc[mm];
                }
        }
    }
}

// ------------------------------------------------------------------------------ bf16 helpers
struct TileRef {
    int seg;       // which weight matrix
    int row0;      // first row of the tile inside that matrix
    int col0;      // first output column of that matrix in the concatenated output
};
__device__ __forceinline__ TileRef find_tile(const GemmArgs &g, int tile, int tile_rows) {
    TileRef t;
    t.seg = 0;
    t.col0 = 0;
    while (t.seg < g.nseg - 1) {
        const int nt = (g.n[t.seg] + tile_rows - 1) / tile_rows;
        if (tile < nt) break;
        tile -= nt;
        t.col0 += g.n[t.seg];
        ++t.seg;
    }
    t.row0 = tile * tile_rows;
    return t;
}

// 8 consecutive activations of one row (zeros for a row past M)
__device__ __forceinline__ f32x8 load_act8(const float *xrow, int k, bool valid) {
    return valid ? load_f32x8(xrow + k) : f32x8{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
}

__device__ __forceinline__ void store_out(const GemmArgs &g, int ks, int m, int col, float v) {
    g.partial[((size_t)ks * g.M + m) * g.N + col] = v;
}



// reduced[m][:] = (sum over splits, in split order) * r_m; one row per blockIdx.y
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(GemmArgs g) {
    __shared__ float red[4];
    const int m = blockIdx.y;
    float sc = 1.0f;
    if (g.scale.sumsq) {
        const size_t src = x_row(g, m);
        float v = 0.f;
        for (int t = threadIdx.x; t < g.scale.tiles; t += 256) v += g.scale.sumsq[(size_t)t * g.scale_rows + src];
        v = wave_sum(v);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        sc = 1.0f / sqrtf((((red[0] + red[1]) + red[2]) + red[3]) * g.scale.inv_d + g.scale.eps);
    }
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col >= g.N) return;
    const size_t idx = (size_t)m * g.N + col;
    float v = 0.f;
    for (int ks = 0; ks < g.splitk; ++ks) v += g.partial[(size_t)ks * g.M * g.N + idx];
    g.reduced[idx] = v * sc;
}

// ------------------------------------------------------------------------------ bf16 skinny
// Block = 4 wavefronts, one 64-row tile of W (4 strips of 16 rows per wavefront, all four
// wavefronts on the same rows, each on its own K range).  Per 128-wide K step a lane issues
// 16 independent 16-byte loads of W (4 strips x 4) and keeps the next step's loads in flight
// while the current one feeds the MFMAs.  The K index inside a step is permuted so that a
// lane's four loads of one row are 2 x 32 contiguous bytes and the four lane groups of a row
// cover 2 x 128 contiguous bytes; the activation operand uses the same permutation.
constexpr int kSkinnyRows = 64;
constexpr int kSkinnyStepK = 128;
constexpr int kStreamBlocks = 512;                 // persistent grid of the unit kernel: 2 blocks per CU

template <int MT>
__global__ __launch_bounds__(256) void gemm_bf16_skinny_kernel(GemmArgs g) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, gq = lane >> 4;
    const TileRef t = find_tile(g, blockIdx.x, kSkinnyRows);
    const int seg_rows = g.n[t.seg];
    const uint16_t *W = (const uint16_t *)g.w[t.seg];
    const float *X = (const float *)g.x;
    const int K = g.K;

    const int nsteps = K / kSkinnyStepK;
    const int S = g.splitk * 4, slot = blockIdx.y * 4 + wave;
    const int s0 = (int)((long)slot * nsteps / S), s1 = (int)((long)(slot + 1) * nsteps / S);

    const uint16_t *wp[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int r = min(t.row0 + s * 16 + i, seg_rows - 1);
        wp[s] = W + (size_t)r * K + gq * 16;
    }
    const float *xp[MT];
    bool xvalid[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int tok = mt * 16 + i;
        xvalid[mt] = tok < g.M;
        xp[mt] = X + x_row(g, min(tok, g.M - 1)) * K + gq * 16;
    }

    f32x4 acc[4][MT];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[s][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    bf16x8 a_cur[4][4], a_nxt[4][4];
    auto load_a = [&](bf16x8 (&dst)[4][4], int step) {
        const int kk = step * kSkinnyStepK;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q) dst[s][q] = *reinterpret_cast<const bf16x8 *>(wp[s] + kk + (q >> 1) * 64 + (q & 1) * 8);
    };
    if (s0 < s1) load_a(a_cur, s0);
    for (int step = s0; step < s1; ++step) {
        if (step + 1 < s1) load_a(a_nxt, step + 1);
        const int kk = step * kSkinnyStepK;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x8 bh[MT], bl[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int k = kk + (q >> 1) * 64 + (q & 1) * 8;
                const f32x8 xv = load_act8(xp[mt], k, xvalid[mt]);
                split_bf16(xv, &bh[mt], &bl[mt]);
            }
            // hi parts over all accumulators, then lo parts: no back-to-back MFMAs on one accumulator
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[s][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_cur[s][q], bh[mt], acc[s][mt], 0, 0, 0);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[s][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_cur[s][q], bl[mt], acc[s][mt], 0, 0, 0);
        }
        if (step + 1 < s1) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int q = 0; q < 4; ++q) a_cur[s][q] = a_nxt[s][q];
        }
    }

    // acc[s][mt][v] = y[token mt*16 + i][row0 + s*16 + 4*gq + v]: add the four wavefronts (K split)
    __shared__ float red[4][kSkinnyRows][17];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (mt) __syncthreads();
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][s * 16 + 4 * gq + v][i] = acc[s][mt][v];
        __syncthreads();
        const int nn = threadIdx.x & 63;
        const int row = t.row0 + nn;
        if (row < seg_rows) {
            for (int mm = threadIdx.x >> 6; mm < 16; mm += 4) {
                const int tok = mt * 16 + mm;
                if (tok < g.M) {
                    const float v = ((red[0][nn][mm] + red[1][nn][mm]) + red[2][nn][mm]) + red[3][nn][mm];
                    store_out(g, blockIdx.y, tok, t.col0 + row, v);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------ bf16 stream-K on packed weights (unit kernel)
// Packed layout of one GEMM (all its weight matrices, in segment order): tiles of 64 rows, each
// tile ns = K/128 units of 16 KB.  Unit = 16 slots of 1 KB, slot index q*4 + strip; slot (q, strip) holds, for
// lane l = (i = l & 15, gq = l >> 4), the 8 bf16 W[tile*64 + strip*16 + i][step*128 + (q>>1)*64 + gq*16 + (q&1)*8 ...]:
// the 4 KB of K quarter q are contiguous.  Rows past the end of a matrix are stored as zeros.
constexpr int kUnitBytes = kSkinnyRows * kSkinnyStepK * 2;
constexpr int kUnitVec = kUnitBytes / 16;          // 16-byte vectors per unit

__global__ __launch_bounds__(256) void gemm_pack_kernel(const uint16_t *W, int N, int K, u32x4 *dst) {
    // one thread per 16-byte vector of the packed copy
    const size_t vec = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int ns = K / kSkinnyStepK;
    const size_t n_units = (size_t)((N + kSkinnyRows - 1) / kSkinnyRows) * ns;
    if (vec >= n_units * kUnitVec) return;
    const size_t unit = vec / kUnitVec;
    const int within = (int)(vec % kUnitVec), slot = within >> 6, lane = within & 63;
    const int tile = (int)(unit / ns), step = (int)(unit % ns);
    const int q = slot >> 2, strip = slot & 3, i = lane & 15, gq = lane >> 4;
    const int row = tile * kSkinnyRows + strip * 16 + i;
    const int k = step * kSkinnyStepK + (q >> 1) * 64 + gq * 16 + (q & 1) * 8;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (row < N) v = *reinterpret_cast<const u32x4 *>(W + (size_t)row * K + k);
    dst[vec] = v;
}

// first unit of block b when U units are dealt to P blocks in contiguous, near-equal ranges
__host__ __device__ __forceinline__ long range_begin(long b, long U, long P) { return b * U / P; }
// the block whose range holds unit u
__host__ __device__ __forceinline__ long range_owner(long u, long U, long P) { return ((u + 1) * P - 1) / U; }

constexpr int kUnitRing = 2;                       // units in flight per wavefront (its 4 KB of each)

// The residual epilogue of one 64-column output tile that several blocks contributed partial sums to.  The calling
// thread holds, for column `col` of the tile (the 64 lanes of its wavefront = the tile's 64 columns), this block's
// sums of rows row0, row0 + rstep, ...: it publishes them in partial slot `slot` with agent-scope stores, waits for
// them, and the block counts itself in on the tile's counter.  Whichever block arrives last adds the tile's
// n_contrib slots in slot order (so the sum does not depend on who that was), adds into the residual stream, writes
// the gain-scaled copy and the rows' sums of squares over the tile, and leaves the counter at zero for the next
// launch.  No block waits for another.  Every thread of the block must call it (it synchronises the block).
template <int NR>
__device__ __forceinline__ void resid_tile_finish(const GemmArgs &g, int tile, int slot, int n_contrib, const float (&mine)[NR],
                                                  int row0, int rstep, bool col_ok, size_t col, int *s_last) {
    bool last = true;
    if (n_contrib > 1) {                                        // the same for the whole block
        if (col_ok)
#pragma unroll
            for (int r = 0; r < NR; ++r)
                if (row0 + r * rstep < g.M)
                    __hip_atomic_store(&g.partial[((size_t)slot * g.M + row0 + r * rstep) * g.N + col], mine[r],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0)
            *s_last = __hip_atomic_fetch_add(&g.tile_counter[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                      (unsigned)(n_contrib - 1);
        __syncthreads();
        last = *s_last != 0;
    }
    if (!last) return;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int tok = row0 + r * rstep;
        float v = 0.f, sq = 0.f;
        if (tok < g.M && col_ok) {
            if (n_contrib > 1) {
                for (int sl = 0; sl < n_contrib; ++sl)
                    v += __hip_atomic_load(&g.partial[((size_t)sl * g.M + tok) * g.N + col], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
            } else {
                v = mine[r];
            }
            const size_t o = (size_t)tok * g.N + col;
            v += g.x_resid[o];
            g.x_resid[o] = v;
            if (g.xg_out) {
                const float xg = v * (g.gain ? bf16_bits_to_f32(((const uint16_t *)g.gain)[col]) : 1.0f);
                g.xg_out[o] = xg;
                if (g.xg16_out) g.xg16_out[o] = f32_to_f16_bits(xg);
            }
            sq = v * v;
        }
        sq = wave_sum(sq);                                      // the tile's 64 columns of row tok sit in this wavefront
        if ((threadIdx.x & 63) == 0 && tok < g.M && g.sumsq_out) g.sumsq_out[(size_t)tile * g.M + tok] = sq;
    }
    if (n_contrib > 1 && threadIdx.x == 0)
        __hip_atomic_store(&g.tile_counter[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A block of a unit kernel is done with a tile (the tile's last unit, or the end of the block's range): red[q][row][token]
// holds the sums of its four wavefronts.  They are added in wavefront order and the block writes ONE partial, slot =
// its index among the blocks that share the tile (the block that finishes the tile zeroes the slots nobody writes),
// or, RESID, hands them to the arrival epilogue above.  upt = units per tile, U = units of the GEMM, P = blocks.
template <bool RESID>
__device__ __forceinline__ void unit_tile_flush(const GemmArgs &g, const float (&red)[4][kSkinnyRows][17], int tile, int upt,
                                                long U, long P, bool tile_end, int *s_last) {
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const TileRef t = find_tile(g, tile, kSkinnyRows);
    const long first_owner = range_owner((long)tile * upt, U, P);
    const int slot = (int)(blockIdx.x - first_owner);
    const int row = t.row0 + lane;                                  // lane = row of the tile
    const bool row_ok = row < g.n[t.seg];
    const size_t col = (size_t)t.col0 + row;
    if constexpr (RESID) {
        const int n_contrib = (int)(range_owner((long)tile * upt + upt - 1, U, P) - first_owner) + 1;
        float mine[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int tok = q + 4 * r;
            mine[r] = ((red[0][lane][tok] + red[1][lane][tok]) + red[2][lane][tok]) + red[3][lane][tok];
        }
        resid_tile_finish<4>(g, tile, slot, n_contrib, mine, q, 4, row_ok, col, s_last);
    } else if (row_ok) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int tok = q + 4 * r;
            if (tok < g.M) {
                g.partial[((size_t)slot * g.M + tok) * g.N + col] =
                    ((red[0][lane][tok] + red[1][lane][tok]) + red[2][lane][tok]) + red[3][lane][tok];
                if (tile_end)
                    for (int jj = slot + 1; jj < g.splitk; ++jj) g.partial[((size_t)jj * g.M + tok) * g.N + col] = 0.f;
            }
        }
    }
}

// Block b streams the contiguous units [range_begin(b), range_begin(b + 1)); wavefront q multiplies the q-th 4 KB of
// every unit (K offsets (q>>1)*64 + (q&1)*8 + 16 gq of the unit's 128), so the four wavefronts of a block read 16 KB
// in one piece and the blocks of the grid adjacent ranges: the access pattern of a plain streaming read.  Weights
// and the matching 8 activations per lane travel through a ring of kUnitRing register stages filled by buffer
// loads: the block's range is the buffer, so the loads issued past its end return zeros without touching memory,
// every wavefront runs the same straight-line loop, and a stage's data is waited for with the later stages still
// in flight.  At the end of a tile (or of the range) the four K quarters are added through LDS in wavefront order
// and the block writes ONE partial: slot = its index among the blocks that share the tile; the block that
// finishes a tile zeroes the slots nobody writes.
//
// RESID (the projections that write the residual stream, when a block per 16 columns would be the slower choice):
// every output element still gets one owner, found at run time.  A block publishes its partial with agent-scope
// stores, waits for them, and counts itself in on the tile's counter; whichever block arrives last adds the tile's
// slots in slot order (so the sum does not depend on who that was) and runs the column kernel's epilogue on the
// tile's 64 columns: residual add, gain-scaled copy, sum of squares per row into sumsq_out[tile][m].  It leaves the
// counter at zero for the next launch.  No block waits for another.
template <bool RESID>
__global__ __launch_bounds__(256) void gemm_bf16_unit_kernel(GemmArgs g) {
    constexpr int R = kUnitRing;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int i = lane & 15, gq = lane >> 4;
    const int K = g.K, ns = K / kSkinnyStepK;
    const long U = (long)g.pack_tiles * ns, P = gridDim.x;
    const int u0 = (int)range_begin(blockIdx.x, U, P), u1 = (int)range_begin(blockIdx.x + 1, U, P);
    if (u0 >= u1) return;
    const int n_my = u1 - u0;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        (char *)const_cast<void *>(g.wpack) + (size_t)u0 * kUnitBytes, 0, n_my * kUnitBytes, 0x00020000);
    // activations: offsets from the first row's source row; a row past M points past the buffer and reads zeros
    const size_t row_first = x_row(g, 0);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(g.x) + row_first * K, 0, 0x7ffffff0, 0x00020000);
    const unsigned kq = (unsigned)((q >> 1) * 64 + gq * 16 + (q & 1) * 8) * 4u;
    const unsigned xbase = i < g.M ? (unsigned)((x_row(g, i) - row_first) * K * 4) + kq : 0x80000000u;

    u32x4 A[R][4], X[R][2];
    int step_issue = u0 % ns;
    auto issue = [&](int j, int n) {                       // n = index of the unit inside the block's range
        const unsigned woff = (unsigned)n * kUnitBytes + q * 4096u + lane * 16u;
#pragma unroll
        for (int s = 0; s < 4; ++s) A[j][s] = __builtin_amdgcn_raw_buffer_load_b128(rw, woff + s * 1024, 0, 2);   // 2: streaming
        const unsigned xoff = n < n_my ? xbase + (unsigned)step_issue * (kSkinnyStepK * 4) : 0x80000000u;
        X[j][0] = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff, 0, 0);
        X[j][1] = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff + 16, 0, 0);
        step_issue = step_issue + 1 == ns ? 0 : step_issue + 1;
    };
    f32x4 acc[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    __shared__ float red[4][kSkinnyRows][17];
    __shared__ int s_last;
#pragma unroll
    for (int j = 0; j < R; ++j) issue(j, j);
    int step_use = u0 % ns, tile = u0 / ns;
    for (int base = 0; base < n_my; base += R) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int n = base + j;
            f32x8 xv;
#pragma unroll
            for (int e = 0; e < 4; ++e) { xv[e] = __uint_as_float(X[j][0][e]); xv[4 + e] = __uint_as_float(X[j][1][e]); }
            bf16x8 bh, bl;
            split_bf16(xv, &bh, &bl);
            // hi parts over all accumulators, then lo parts: no back-to-back MFMAs on one accumulator
#pragma unroll
            for (int s = 0; s < 4; ++s)
                acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[j][s]), bh, acc[s], 0, 0, 0);
#pragma unroll
            for (int s = 0; s < 4; ++s)
                acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[j][s]), bl, acc[s], 0, 0, 0);
            issue(j, n + R);
            const bool tile_end = step_use + 1 == ns;
            step_use = tile_end ? 0 : step_use + 1;
            if (n < n_my && (tile_end || n + 1 == n_my)) {                  // the same for all four wavefronts
                // acc[s][v] = y[token i][row s*16 + 4*gq + v of the tile] over this wavefront's K quarter
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int v = 0; v < 4; ++v) red[q][s * 16 + 4 * gq + v][i] = acc[s][v];
                __syncthreads();
                unit_tile_flush<RESID>(g, red, tile, ns, U, P, tile_end, &s_last);
                __syncthreads();
#pragma unroll
                for (int s = 0; s < 4; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            if (tile_end) ++tile;
        }
    }
}

// ------------------------------------------------------------------------------ bf16 one-slot column kernel
// For the projections that write the residual stream (N = d_model): one block per 16 output columns over
// the whole K range, its wavefronts (sixteen for up to 16 rows, eight above: registers) on different K ranges, added through LDS in wavefront order.
// Every output element has a single owner, so the block finishes the job itself: x_resid[m][n] += y[m][n],
// xg_out[m][n] = x_resid[m][n] * gain_next[n] (the operand of the next projection, RMSNorm gain folded in),
// and the sum of squares of the updated 16 columns per row goes to sumsq_out, from which the consumer of the
// next projection derives the RMSNorm scale.  No partial slots, no reduce kernel, no norm kernel.
// Weights are packed strip-major for this kernel (gemm_pack_strip_kernel): strip (16 rows) x K step is 4 KB
// = 4 slots of 1 KB in lane order, all K steps of a strip contiguous, so a block streams one contiguous
// range and a wavefront a contiguous part of it, 16 KB in flight at a time.
constexpr int kColDepth = 4;                       // K steps loaded per round
constexpr int kStripVec = 16 * kSkinnyStepK * 2 / 16;   // 16-byte vectors per (strip, step)

__global__ __launch_bounds__(256) void gemm_pack_strip_kernel(const uint16_t *W, int N, int K, u32x4 *dst) {
    const size_t vec = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int ns = K / kSkinnyStepK;
    const size_t strips = (size_t)((N + kSkinnyRows - 1) / kSkinnyRows) * 4;
    if (vec >= strips * ns * kStripVec) return;
    const size_t strip = vec / ((size_t)ns * kStripVec);
    const int rem = (int)(vec % ((size_t)ns * kStripVec));
    const int step = rem / kStripVec, q = (rem % kStripVec) >> 6, lane = rem & 63;
    const int i = lane & 15, gq = lane >> 4;
    const size_t row = strip * 16 + i;
    const int k = step * kSkinnyStepK + (q >> 1) * 64 + gq * 16 + (q & 1) * 8;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (row < (size_t)N) v = *reinterpret_cast<const u32x4 *>(W + row * K + k);
    dst[vec] = v;
}

// 4-bit weights (W4A16, asymmetric, groups of 128 along K = one K step): w = scale * (q - zero).  Packed layout
// of one GEMM: tiles of 64 rows, each tile ceil(ns / 4) quads, a quad = four consecutive K steps of the tile
// (K steps past the end of K are stored with scale 0), a step = 4352 bytes: four 1 KB slots of codes, one per
// strip of 16 rows, in lane order (lane (n, gq) owns one 16-byte vector: dword kb holds its eight nibbles of row
// strip*16 + n, K offsets kb*32 + gq*8 ..+7 of the step, element e at bit 4*(e/2) + 16*(e&1), so that
// (dword >> 4p) & 0x000F000F is the element pair (2p, 2p+1)), then 256 bytes of scales and zero points: the word
// of (row n, strip s) at [n][s] holds the bf16 scale in its high half and the fp16 number 1024 + zero (bit
// pattern 0x6400 | zero) in its low half.  The kernel multiplies the nibbles as the exact fp16 integers
// 1024 + q (bit pattern 0x6400 | q) and takes scale * (sum (1024 + q) x - (1024 + zero) sum x) per group, so
// no weight is ever rounded.
constexpr int kW4StepBytes = 4096 + 256;
constexpr int kW4QuadBytes = 4 * kW4StepBytes;
__host__ __device__ __forceinline__ int w4_quads(int K) { return (K / kSkinnyStepK + 3) / 4; }

__global__ __launch_bounds__(64) void gemm_pack_w4_kernel(const uint8_t *Q, const uint16_t *scale, const uint8_t *zero,
                                                          int N, int K, uint8_t *dst) {
    // one block per stored K step: blockIdx.x = tile * (4 * quads) + step
    const int ns = K / kSkinnyStepK, ns4 = 4 * w4_quads(K);
    const size_t tile = blockIdx.x / ns4;
    const int step = blockIdx.x % ns4, lane = threadIdx.x, n = lane & 15, gq = lane >> 4;
    uint8_t *out = dst + (size_t)blockIdx.x * kW4StepBytes;
#pragma unroll
    for (int strip = 0; strip < 4; ++strip) {
        const size_t row = tile * kSkinnyRows + strip * 16 + n;
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (row < (size_t)N && step < ns) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const int k = step * kSkinnyStepK + kb * 32 + gq * 8;
                const uint32_t raw = *reinterpret_cast<const uint32_t *>(Q + (row * K + k) / 2);   // byte b: k + 2b, k + 2b + 1
                uint32_t w = 0;
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) {
                    w |= ((raw >> (8 * bb)) & 0xFu) << (4 * bb);                // element 2 bb
                    w |= ((raw >> (8 * bb + 4)) & 0xFu) << (16 + 4 * bb);       // element 2 bb + 1
                }
                v[kb] = w;
            }
        }
        reinterpret_cast<u32x4 *>(out + strip * 1024)[lane] = v;
    }
    {
        const int strip = lane >> 4;
        const size_t row = tile * kSkinnyRows + strip * 16 + n;
        uint32_t sz = 0x6400u;                                                   // rows and steps past the end: scale 0
        if (row < (size_t)N && step < ns)
            sz = ((uint32_t)scale[row * ns + step] << 16) | (0x6400u | zero[row * ns + step]);   // zero <= 15
        reinterpret_cast<uint32_t *>(out + 4096)[n * 4 + strip] = sz;
    }
}

template <int MT, int kColWaves>
__global__ __launch_bounds__(kColWaves * 64) void gemm_bf16_column_kernel(GemmArgs g) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, gq = lane >> 4;
    const int K = g.K, ns = K / kSkinnyStepK;
    const int s0 = wave * ns / kColWaves, s1 = (wave + 1) * ns / kColWaves;

    // the epilogue's operands, fetched before the main loop: thread t < 256 owns column n = t & 15 of rows mm = t >> 4
    const int en = threadIdx.x & 15, emm = threadIdx.x >> 4;
    const int ecol = blockIdx.x * 16 + en;
    float e_res[MT], e_gain = 1.0f;
    if (threadIdx.x < 256 && ecol < g.N) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int tok = mt * 16 + emm;
            e_res[mt] = tok < g.M && g.x_resid ? g.x_resid[(size_t)tok * g.N + ecol] : 0.f;
        }
        if (g.gain) e_gain = bf16_bits_to_f32(((const uint16_t *)g.gain)[ecol]);
    }

    const float *xp[MT];
    bool xvalid[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int tok = mt * 16 + i;
        xvalid[mt] = tok < g.M;
        xp[mt] = g.x + x_row(g, min(tok, g.M - 1)) * K + gq * 16;
    }
    f32x4 acc[2][MT];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[h][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const u32x4 *wbase = reinterpret_cast<const u32x4 *>(g.wpack) + (size_t)blockIdx.x * ns * kStripVec + lane;
    for (int step = s0; step < s1; step += kColDepth) {
        u32x4 a[kColDepth * 4];
#pragma unroll
        for (int j = 0; j < kColDepth; ++j)
            if (step + j < s1) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    a[j * 4 + q] = __builtin_nontemporal_load(wbase + (size_t)(step + j) * kStripVec + q * 64);
            }
#pragma unroll
        for (int j = 0; j < kColDepth; ++j) {
            if (step + j >= s1) break;
            f32x8 xv[4][MT];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    xv[q][mt] = load_act8(xp[mt], (step + j) * kSkinnyStepK + (q >> 1) * 64 + (q & 1) * 8, xvalid[mt]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bf16x8 aw = __builtin_bit_cast(bf16x8, a[j * 4 + q]);
                bf16x8 bh[MT], bl[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) split_bf16(xv[q][mt], &bh[mt], &bl[mt]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[q & 1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw, bh[mt], acc[q & 1][mt], 0, 0, 0);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[q & 1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw, bl[mt], acc[q & 1][mt], 0, 0, 0);
            }
        }
    }

    // acc[.][mt][v] = y[token mt*16 + i][column 4*gq + v of the strip] over this wavefront's K steps
    __shared__ float red[kColWaves][16][17];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (mt) __syncthreads();
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][4 * gq + v][i] = acc[0][mt][v] + acc[1][mt][v];
        __syncthreads();
        if (threadIdx.x < 256) {
            const int tok = mt * 16 + emm;
            float v = 0.f, sq = 0.f;
#pragma unroll
            for (int w = 0; w < kColWaves; ++w) v += red[w][en][emm];
            if (tok < g.M && ecol < g.N) {
                const size_t o = (size_t)tok * g.N + ecol;
                if (g.x_resid) {
                    v += e_res[mt];
                    g.x_resid[o] = v;
                    if (g.xg_out) g.xg_out[o] = v * e_gain;
                    sq = v * v;
                } else {
                    g.partial[o] = v;                        // one slot: the projection's output itself
                }
            }
            // the 16 columns of one row sit in 16 consecutive lanes
            sq += __shfl_xor(sq, 8, 64);
            sq += __shfl_xor(sq, 4, 64);
            sq += __shfl_xor(sq, 2, 64);
            sq += __shfl_xor(sq, 1, 64);
            if (en == 0 && tok < g.M && g.sumsq_out) g.sumsq_out[(size_t)blockIdx.x * g.M + tok] = sq;
        }
    }
}

// ------------------------------------------------------------------------------ 4-bit weights, M <= 16
// The unit kernel's scheme on the 4-bit layout: the unit is a quad (four K steps of a 64-row tile, 17 KB), block b
// streams the contiguous quads [range_begin(b), range_begin(b + 1)), wavefront q multiplies step q of every quad
// (its 4352 contiguous bytes), the four wavefronts' sums meet in LDS at the end of a tile, one partial slot per
// block and tile or the arrival epilogue (O, down).  Codes, scales and activations travel through a ring of
// register stages filled by buffer loads that return zeros past the end of the block's range.
// The activations are the MFMA's row operand here and the weights its column operand, so that a lane holds four
// tokens of ONE weight row per strip and applies that row's scale and zero point as two scalars per group:
// u = sum (1024 + q) x on the matrix cores with the codes as exact fp16 integers, xs = sum x with an all-ones
// operand, then acc += scale * (u - (1024 + zero) * xs) in fp32.  The activations are read from the fp16 copy their
// producers leave beside the fp32 ones (11 significant bits, as for the tiled kernel; activations beyond +-65504
// would overflow): half the bytes every block re-reads from L2, which weigh as much as the 4-bit weights themselves.
constexpr int kW4Ring = 2;                         // quads in flight per wavefront (its K step of each)

template <bool RESID>
__global__ __launch_bounds__(256) void gemm_w4_unit_kernel(GemmArgs g) {
    constexpr int R = kW4Ring;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int i = lane & 15, gq = lane >> 4;
    const int K = g.K, ns = K / kSkinnyStepK, nq = w4_quads(K);
    const long U = (long)g.pack_tiles * nq, P = gridDim.x;
    const int u0 = (int)range_begin(blockIdx.x, U, P), u1 = (int)range_begin(blockIdx.x + 1, U, P);
    if (u0 >= u1) return;
    const int n_my = u1 - u0;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        (char *)const_cast<void *>(g.wpack) + (size_t)u0 * kW4QuadBytes, 0, n_my * kW4QuadBytes, 0x00020000);
    // activations (the fp16 copy): offsets from the first row's source row; a row past M points past the buffer and
    // reads zeros.  Lane (token i, gq) multiplies K offsets kb*32 + gq*8 ..+7 of its step in MFMA kb.
    const size_t row_first = x_row(g, 0);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(g.x16) + row_first * K, 0, 0x7ffffff0, 0x00020000);
    const unsigned xbase = i < g.M ? (unsigned)((x_row(g, i) - row_first) * K * 2) + gq * 16u : 0x80000000u;

    u32x4 C[R][4], S[R], X[R][4];
    int quad_issue = u0 % nq;
    auto issue = [&](int j, int n) {                       // n = index of the quad inside the block's range
        const unsigned woff = (unsigned)n * kW4QuadBytes + q * kW4StepBytes;
#pragma unroll
        for (int s = 0; s < 4; ++s) C[j][s] = __builtin_amdgcn_raw_buffer_load_b128(rw, woff + s * 1024 + lane * 16u, 0, 2);   // 2: streaming
        S[j] = __builtin_amdgcn_raw_buffer_load_b128(rw, woff + 4096 + i * 16u, 0, 2);
        const int step = quad_issue * 4 + q;
        const unsigned xoff = n < n_my && step < ns ? xbase + (unsigned)step * (kSkinnyStepK * 2) : 0x80000000u;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) X[j][kb] = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff + kb * 64, 0, 0);
        quad_issue = quad_issue + 1 == nq ? 0 : quad_issue + 1;
    };
    const u32x4 ones4 = u32x4{0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
    const f16x8 ones = __builtin_bit_cast(f16x8, ones4);
    f32x4 acc[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    __shared__ float red[4][kSkinnyRows][17];
    __shared__ int s_last;
#pragma unroll
    for (int j = 0; j < R; ++j) issue(j, j);
    int quad_use = u0 % nq, tile = u0 / nq;
    for (int base = 0; base < n_my; base += R) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int n = base + j;
            if (n >= n_my) break;                                           // the same for all four wavefronts
            f32x4 u[4], xs = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) u[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const f16x8 xa = __builtin_bit_cast(f16x8, X[j][kb]);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint32_t w = C[j][s][kb];
                    const u32x4 wi = u32x4{(w & 0x000F000Fu) | 0x64006400u, ((w >> 4) & 0x000F000Fu) | 0x64006400u,
                                           ((w >> 8) & 0x000F000Fu) | 0x64006400u, ((w >> 12) & 0x000F000Fu) | 0x64006400u};
                    u[s] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa, __builtin_bit_cast(f16x8, wi), u[s], 0, 0, 0);
                }
                xs = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa, ones, xs, 0, 0, 0);       // sum of x over the group
            }
            // u[s][v] = sum over the group of x[token 4 gq + v] * (1024 + q[row s*16 + i]); xs[v] = sum of x[token 4 gq + v]
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const uint32_t sz = S[j][s];
                const float sc = __uint_as_float(sz & 0xffff0000u);
                const float zf = (float)__builtin_bit_cast(_Float16, (uint16_t)(sz & 0xffffu));
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[s][v] += sc * (u[s][v] - zf * xs[v]);
            }
            issue(j, n + R);
            const bool tile_end = quad_use + 1 == nq;
            quad_use = tile_end ? 0 : quad_use + 1;
            if (tile_end || n + 1 == n_my) {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int v = 0; v < 4; ++v) red[q][s * 16 + i][4 * gq + v] = acc[s][v];
                __syncthreads();
                unit_tile_flush<RESID>(g, red, tile, nq, U, P, tile_end, &s_last);
                __syncthreads();
#pragma unroll
                for (int s = 0; s < 4; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            if (tile_end) ++tile;
        }
    }
}

typedef __attribute__((ext_vector_type(2))) uint32_t uint2v;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
// 8 four-bit codes (element e in bits 4e .. 4e+3) -> 8 fp16 weights scale * (q - zero); sz = fp16 scale in the high
// half, fp16 1024 + zero in the low half
__device__ __forceinline__ u32x4 w4x8_to_f16x8(uint32_t raw, uint32_t sz) {
    const _Float16 zf = __builtin_bit_cast(_Float16, (uint16_t)(sz & 0xffffu));
    const _Float16 sf = __builtin_bit_cast(_Float16, (uint16_t)(sz >> 16));
    const f16x2 z2 = f16x2{zf, zf}, s2 = f16x2{sf, sf};
    u32x4 r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t t = raw >> (8 * p);
        const uint32_t pair = (t & 0xFu) | ((t & 0xF0u) << 12) | 0x64006400u;   // fp16 1024 + q of elements 2p, 2p+1
        r[p] = __builtin_bit_cast(uint32_t, (__builtin_bit_cast(f16x2, pair) - z2) * s2);
    }
    return r;
}

// ------------------------------------------------------------------------------ tiled (M > 16)
// Block tile 128 or 256 rows of activations x 32*NB rows of W x 64 of K (NB = 4, 6, 8); wavefronts in a 2 x 2 or
// 4 x 2 grid, each on 64 activation rows x 16*NB weight rows: 2 x NB/2 tiles of the 32x32x16 MFMA, so that per 16-wide K step
// a wavefront reads 2 + NB/2 operands from LDS for NB MFMAs (with 1 x NB tiles per wavefront it would be 1 + NB
// operands, and LDS reads, not the matrix cores, would set the pace).
// Both operands enter the matrix cores as fp16, one product each: the bf16 weights convert to fp16 exactly
// (8 significant bits into 11; only magnitudes below 7.6e-6 fall under the fp16 grid and are rounded to it, by at
// most 3e-8), the fp32 activations are rounded to fp16 (11 significant bits, the error of bf16 divided by 8),
// which keeps the logits of the 7B-shaped models within 2e-2 of the fp64 result at half the MFMA issue of a
// bf16 high + low pair.  Activations beyond +-65504 would overflow; none of the decoder's normalised or gated
// activations come near.  Rows are padded to 72 elements (144 B): conflict-free 16-byte reads.  LDS is dynamic.
// 128-row blocks run two per CU (one block's staging and barriers overlap the other's MFMAs); 256-row blocks run
// one per CU with two sets of LDS tiles and two K tiles in flight in registers (what a CU keeps in flight bounds
// its load rate, and one K tile is too little of it).
// The tile width and the K split are chosen per projection by the host so that the number of blocks comes
// close to a multiple of the resident block slots.
constexpr int kBK = 64, kLdsStride = 72, kMaxNB = 8;
constexpr int kTallRows = 160;                           // from this many rows on: 256-row blocks
inline int tiled_block_rows(int M) { return M >= kTallRows ? 256 : 128; }

// MW = wavefront rows of the block: 2 (128 activation rows, 256 threads, two blocks per CU) or 4 (256 rows, 512
// threads, one block per CU: each weight tile then leaves L2 once for 256 rows instead of twice).
// W4: the weights are 4-bit codes as the caller stores them (row-major, low nibble = even k) with a bf16 scale and
// a zero point per row and group of 128 k.  A thread's 8 weights of a K tile are 4 bytes of codes; on the way into
// LDS they become the fp16 numbers scale * (q - zero): (1024 + q) - (1024 + zero) is exact in fp16, the product
// with the scale (itself exact in fp16 down to 6e-5) is rounded once, to 11 significant bits.
template <int NB, int MW, bool W4 = false>
__global__ __launch_bounds__(MW * 128, MW == 2 ? 2 : 1) void gemm_f16_tiled_kernel(GemmArgs g) {
    constexpr int BM = 64 * MW, BN = 32 * NB, NH = NB / 2, NT = MW * 128;
    constexpr int XCH = BM * 8 / NT;                        // 16-byte chunks of the fp16 X tile per thread (BM x 64)
    constexpr int WCH = BN * 8 / NT;                        // 16-byte chunks of the W tile per thread (BN x 64 bf16)
    // MW == 4 has the CU to itself and LDS for two sets of tiles: the next K tile is stored into the other set in
    // the middle of this tile's MFMAs (one barrier per K tile, no phase in which the matrix cores wait for the
    // stores).  MW == 2 keeps one set: two blocks share the CU and overlap each other's barriers.
    constexpr bool DB = MW == 4;
    constexpr int kSet = (BM + BN) * kLdsStride;            // elements of one set of tiles
    extern __shared__ __attribute__((aligned(16))) uint16_t lds_tiled[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * (BN / 2);   // this wavefront's corner of the block tile
    const int m_tiles = (g.M + BM - 1) / BM;
    const int mt = blockIdx.x % m_tiles;                 // M tiles of one W tile are neighbours: W is re-read from L2
    const TileRef t = find_tile(g, blockIdx.x / m_tiles, BN);
    const int seg_rows = g.n[t.seg];
    const uint16_t *W = (const uint16_t *)g.w[t.seg];
    const int K = g.K;
    const int nk = K / kBK;
    const int k0 = (int)((long)blockIdx.y * nk / g.splitk), k1 = (int)((long)(blockIdx.y + 1) * nk / g.splitk);
    const int m_base = mt * BM;

    // global -> register staging per K tile: XCH x 8 activations (fp16 copy if there is one, else fp32 rounded
    // here) and WCH x 8 bf16 of W per thread
    uint32_t xsrc[XCH], wsrc[WCH];                       // element offsets from the matrices' first elements
    uint32_t wgrp[WCH];                                  // W4: index of the row's first group in scale / zero
    int xoff[XCH], woff[WCH];
#pragma unroll
    for (int c = 0; c < XCH; ++c) {
        const int chunk = tid + c * NT, row = chunk >> 3, col = (chunk & 7) * 8;
        xsrc[c] = (uint32_t)(x_row(g, min(m_base + row, g.M - 1)) * K + col);
        xoff[c] = row * kLdsStride + col;
    }
#pragma unroll
    for (int c = 0; c < WCH; ++c) {
        const int chunk = tid + c * NT, row = chunk >> 3, col = (chunk & 7) * 8;
        wsrc[c] = (uint32_t)((size_t)min(t.row0 + row, seg_rows - 1) * K + col);
        wgrp[c] = (uint32_t)(min(t.row0 + row, seg_rows - 1) * (K / kSkinnyStepK));
        woff[c] = row * kLdsStride + col;
    }
    const uint8_t *Wq = (const uint8_t *)g.w[t.seg];
    const uint16_t *Wscale = (const uint16_t *)g.w4_scale[t.seg];
    const uint8_t *Wzero = (const uint8_t *)g.w4_zero[t.seg];
    const bool have16 = g.x16 != nullptr;
    // Register stages of the global -> LDS path.  What one CU keeps in flight bounds its load rate (bytes in flight /
    // latency), and one K tile per block is too little of it: with two sets of LDS tiles the block also keeps two
    // K tiles in flight in registers (stage = tile parity), except at the widest tile where the registers run out.
    constexpr int NST = (DB && NB <= 6) ? 2 : 1;
    using WReg = std::conditional_t<W4, uint2v, u32x4>;   // what a thread holds of one 8-weight chunk
    u32x4 xr[NST][XCH];
    WReg wr[NST][WCH];
    auto load_tiles = [&](auto stage, int kt) {
        constexpr int st = decltype(stage)::value;
#pragma unroll
        for (int c = 0; c < XCH; ++c) {
            if (have16) xr[st][c] = *reinterpret_cast<const u32x4 *>(g.x16 + xsrc[c] + kt * kBK);
            else xr[st][c] = f32x8_to_f16x8(load_f32x8(g.x + xsrc[c] + kt * kBK));
        }
#pragma unroll
        for (int c = 0; c < WCH; ++c) {
            if constexpr (W4) {
                // [0]: the 8 codes; [1]: fp16 scale (high half) and fp16 1024 + zero (low half) of the row's group
                const uint32_t grp = wgrp[c] + (uint32_t)(kt * kBK / kSkinnyStepK);
                const _Float16 sc = (_Float16)bf16_bits_to_f32(Wscale[grp]);
                wr[st][c][0] = *reinterpret_cast<const uint32_t *>(Wq + (wsrc[c] + kt * kBK) / 2);
                wr[st][c][1] = ((uint32_t)__builtin_bit_cast(uint16_t, sc) << 16) | 0x6400u | Wzero[grp];
            } else {
                wr[st][c] = *reinterpret_cast<const u32x4 *>(W + wsrc[c] + kt * kBK);
            }
        }
    };
    auto store_tiles = [&](auto stage, int set) {
        constexpr int st = decltype(stage)::value;
        uint16_t *Xs = lds_tiled + set * kSet, *Ws = Xs + BM * kLdsStride;     // activation tile, weight tile (fp16)
#pragma unroll
        for (int c = 0; c < XCH; ++c) *reinterpret_cast<u32x4 *>(&Xs[xoff[c]]) = xr[st][c];
#pragma unroll
        for (int c = 0; c < WCH; ++c) {
            if constexpr (W4) *reinterpret_cast<u32x4 *>(&Ws[woff[c]]) = w4x8_to_f16x8(wr[st][c][0], wr[st][c][1]);
            else *reinterpret_cast<u32x4 *>(&Ws[woff[c]]) = bf16x8_to_f16x8(wr[st][c]);
        }
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, NST - 1>;      // the second stage, or the only one

    f32x16 acc[2][NH];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NH; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    auto multiply = [&](int set, int ks) {
        const uint16_t *Xs = lds_tiled + set * kSet, *Ws = Xs + BM * kLdsStride;
        f16x8 fa[2], fb[NH];
#pragma unroll
        for (int a = 0; a < 2; ++a)
            fa[a] = *reinterpret_cast<const f16x8 *>(&Xs[(wm + a * 32 + li) * kLdsStride + ks * 16 + lg * 8]);
#pragma unroll
        for (int b = 0; b < NH; ++b)
            fb[b] = *reinterpret_cast<const f16x8 *>(&Ws[(wn + b * 32 + li) * kLdsStride + ks * 16 + lg * 8]);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < NH; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    };
    if (k0 < k1) {
        load_tiles(S0{}, k0);
        store_tiles(S0{}, 0);
        if constexpr (NST == 2) {
            // tile t travels in stage (t - k0) & 1
            if (k0 + 1 < k1) load_tiles(S1{}, k0 + 1);
            if (k0 + 2 < k1) load_tiles(S0{}, k0 + 2);
        } else if (DB && k0 + 1 < k1) {
            load_tiles(S0{}, k0 + 1);
        }
    }
    __syncthreads();
    if constexpr (DB) {
        // one K tile: half its MFMAs, the next tile from its registers into the other LDS set, the registers refilled
        // with the tile NST ahead, the other half, one barrier (tile kt + 1 visible; this set free for tile kt + 2)
        auto k_tile = [&](auto next_stage, int kt) {
            const int set = (kt - k0) & 1;
            multiply(set, 0);
            multiply(set, 1);
            if (kt + 1 < k1) store_tiles(next_stage, set ^ 1);
            if (kt + 1 + NST < k1) load_tiles(next_stage, kt + 1 + NST);
            multiply(set, 2);
            multiply(set, 3);
            __syncthreads();
        };
        int kt = k0;
        for (; kt + 1 < k1; kt += 2) {
            k_tile(S1{}, kt);                                // tile kt + 1 has odd parity
            k_tile(S0{}, kt + 1);
        }
        if (kt < k1) k_tile(S1{}, kt);
    } else {
        for (int kt = k0; kt < k1; ++kt) {
            if (kt + 1 < k1) load_tiles(S0{}, kt + 1);       // in flight while this tile is multiplied
#pragma unroll
            for (int ks = 0; ks < kBK / 16; ++ks) multiply(0, ks);
            __syncthreads();
            if (kt + 1 < k1) store_tiles(S0{}, 0);
            __syncthreads();
        }
    }
    // acc[a][b][v] = y[m_base + wm + a*32 + 8*(v/4) + 4*lg + v%4][row0 + wn + b*32 + li]
#pragma unroll
    for (int b = 0; b < NH; ++b) {
        const int row = t.row0 + wn + b * 32 + li;
        if (row >= seg_rows) continue;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m_base + wm + a * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                if (m < g.M) store_out(g, blockIdx.y, m, t.col0 + row, acc[a][b][v]);
            }
    }
}

int tiles_of(const int *n, int nseg, int rows) {
    int t = 0;
    for (int s = 0; s < nseg; ++s) t += (n[s] + rows - 1) / rows;
    return t;
}

}  // namespace

// Tile width (NB x 32 columns, NB = 4, 6, 8) and K split of the tiled kernel: the pair with the least estimated
// time: rounds of 512 resident blocks x K tiles per block x the time of one K tile of two co-resident blocks,
// which the LDS traffic sets (16 KB of activations and 4 NB KB of weights written, 4 (2 + NB/2) x 4 KB read, at
// 128 B per clock, with a margin for what does not overlap), plus writing and re-reading one fp32 partial slot of
// M x N per split at about 3 TB/s.
static void tiled_choice(int M, int K, const int *n, int nseg, int *nb_out, int *sk_out) {
    const int bm = tiled_block_rows(M), nk = K / kBK, m_tiles = (M + bm - 1) / bm;
    const int slots = bm == 256 ? 256 : 512;          // resident blocks: one 512-thread or two 256-thread blocks per CU
    long N = 0;
    for (int s = 0; s < nseg; ++s) N += n[s];
    const double slot_us = 2.0 * (double)M * (double)N * 4.0 / 3.0e6;
    double best = 1e300;
    *nb_out = 6; *sk_out = 1;
    for (int nb = 4; nb <= kMaxNB; nb += 2)
        for (int sk = 1; sk <= 16 && (sk == 1 || nk / sk >= 4); ++sk) {
            const long blocks = (long)tiles_of(n, nseg, 32 * nb) * m_tiles * sk;
            const long rounds = (blocks + slots - 1) / slots;
            const double tile_clk = (48.0 + 12.0 * nb) * 8.0 * 1.3;     // per 128 rows
            const double cost = rounds * (double)((nk + sk - 1) / sk) * 2.0 * tile_clk / 2400.0 + sk * slot_us;
            if (cost < best) { best = cost; *nb_out = nb; *sk_out = sk; }
        }
}

int gemm_stream_grid(int tiles, int K) {
    const long U = (long)tiles * (K / kSkinnyStepK);
    return (int)(U < kStreamBlocks ? (U < 1 ? 1 : U) : kStreamBlocks);
}

// grid of the unit kernel with the residual epilogue: one block per CU, so that few blocks share a tile (the last of
// them to arrive adds their partials).  Measured on the 7B down projection, O and down averaged: 256 blocks 16.2 us,
// 384 blocks 18.5 us, 512 blocks 17.8 us, 128 blocks slower still.
int gemm_resid_grid(int tiles, int K) {
    const long U = (long)tiles * (K / kSkinnyStepK);
    return (int)(U < kStreamBlocks / 2 ? (U < 1 ? 1 : U) : kStreamBlocks / 2);
}

// largest number of blocks that share one tile, i.e. partial slots per output element
static int gemm_slots_of(int tiles, int units_per_tile, int grid);
int gemm_resid_slots(int tiles, int K) { return gemm_slots_of(tiles, K / kSkinnyStepK, gemm_resid_grid(tiles, K)); }
int gemm_stream_slots(int tiles, int K) { return gemm_slots_of(tiles, K / kSkinnyStepK, gemm_stream_grid(tiles, K)); }
static int gemm_slots_of(int tiles, int units_per_tile, int grid) {
    const long ns = units_per_tile, U = (long)tiles * ns, P = grid;
    long worst = 1;
    for (long t = 0; t < tiles; ++t) {
        const long span = range_owner((t + 1) * ns - 1, U, P) - range_owner(t * ns, U, P) + 1;
        if (span > worst) worst = span;
    }
    return (int)worst;
}

int gemm_pack_tiles(const int *n, int nseg) { return tiles_of(n, nseg, kSkinnyRows); }
size_t gemm_pack_bytes(const int *n, int nseg, int K) {
    return (size_t)tiles_of(n, nseg, kSkinnyRows) * (K / kSkinnyStepK) * kUnitBytes;
}

void launch_gemm_pack(const void *const *w, const int *n, int nseg, int K, void *dst, bool strip_major, hipStream_t stream) {
    char *out = (char *)dst;
    for (int s = 0; s < nseg; ++s) {
        const size_t units = (size_t)((n[s] + kSkinnyRows - 1) / kSkinnyRows) * (K / kSkinnyStepK);
        const size_t vecs = units * kUnitVec;
        if (strip_major)
            launch_kernel(gemm_pack_strip_kernel, (unsigned)((vecs + 255) / 256), 256, 0, stream, (const uint16_t *)w[s], n[s], K, (u32x4 *)out);
        else
            launch_kernel(gemm_pack_kernel, (unsigned)((vecs + 255) / 256), 256, 0, stream, (const uint16_t *)w[s], n[s], K, (u32x4 *)out);
        out += units * kUnitBytes;
    }
}

size_t gemm_pack_w4_bytes(const int *n, int nseg, int K) {
    return (size_t)tiles_of(n, nseg, kSkinnyRows) * w4_quads(K) * kW4QuadBytes;
}

void launch_gemm_pack_w4(const void *const *q, const void *const *scale, const void *const *zero, const int *n,
                         int nseg, int K, void *dst, hipStream_t stream) {
    uint8_t *out = (uint8_t *)dst;
    const int ns4 = 4 * w4_quads(K);
    for (int s = 0; s < nseg; ++s) {
        const size_t tiles = (size_t)((n[s] + kSkinnyRows - 1) / kSkinnyRows);
        launch_kernel(gemm_pack_w4_kernel, (unsigned)(tiles * ns4), 64, 0, stream, (const uint8_t *)q[s],
                      (const uint16_t *)scale[s], (const uint8_t *)zero[s], n[s], K, out);
        out += tiles * ns4 * kW4StepBytes;
    }
}

// grid and partial slots of a 4-bit projection: the unit kernel's policy with the quad as the unit, except that a
// block gets at least three quads where that still leaves one block per CU (measured on the LLaMA3-8B shape: QKV,
// 768 quads, 8.0 us on 512 blocks and 7.2 us on 256; gate|up, 3584 quads, 15.3 us on 512 and 17.6 us on 256; the
// residual projections 15.4 us (down) on 256 blocks, 16.9 us on 512, 18.9 us on 128)
static int gemm_w4_grid(int tiles, int K, bool resid) {
    const long U = (long)tiles * w4_quads(K);
    long cap = kStreamBlocks / 2;
    if (!resid && U / 3 > cap) cap = U / 3 < kStreamBlocks ? U / 3 : kStreamBlocks;
    return (int)(U < cap ? (U < 1 ? 1 : U) : cap);
}
int gemm_w4_slots(int K, const int *n, int nseg, bool resid) {
    const int tiles = tiles_of(n, nseg, kSkinnyRows);
    return gemm_slots_of(tiles, w4_quads(K), gemm_w4_grid(tiles, K, resid));
}

int gemm_packed_splits(int M, int K, const int *n, int nseg) {
    (void)M;
    return gemm_stream_slots(tiles_of(n, nseg, kSkinnyRows), K);
}

int gemm_pick_splitk(int dtype, int M, int K, int N, const int *n, int nseg) {
    (void)N;
    if (dtype != PSD_BF16) return 1;
    if (M <= kStreamMaxRows) {
        const int tiles = tiles_of(n, nseg, kSkinnyRows);
        const int nsteps = K / kSkinnyStepK;
        int want = (512 + tiles - 1) / tiles;             // aim at >= 512 blocks (2048 wavefronts)
        int cap = nsteps / 8;                             // keep >= 2 K steps per wavefront
        if (cap < 1) cap = 1;
        if (want > cap) want = cap;
        if (want > 16) want = 16;
        return want < 1 ? 1 : want;
    }
    int nb, sk;
    tiled_choice(M, K, n, nseg, &nb, &sk);
    return sk;
}

void launch_gemm(int dtype, const GemmArgs &g, hipStream_t stream) {
    if (dtype != PSD_BF16) {
        ScopedProf sp(PSD_KIND_GEMM_F32, stream);
        launch_kernel(gemm_f32_kernel, (g.N + 3) / 4, 256, 0, stream, g);
        return;
    }
    if (g.M <= kStreamMaxRows && g.wpack && g.w4) {
        // 32-bit offsets from the first activation row: these projections read M <= 16 consecutive rows
        ScopedProf sp(PSD_KIND_GEMM_W4, stream);
        const bool resid = g.x_resid && g.tile_counter;
        const int grid = gemm_w4_grid(g.pack_tiles, g.K, resid);
        if (resid)
            launch_kernel(gemm_w4_unit_kernel<true>, grid, 256, 0, stream, g);
        else
            launch_kernel(gemm_w4_unit_kernel<false>, grid, 256, 0, stream, g);
        return;
    }
    if (g.M <= kStreamMaxRows && g.wpack && g.x_resid && g.tile_counter) {
        ScopedProf sp(PSD_KIND_GEMM_COLUMN, stream);
        launch_kernel(gemm_bf16_unit_kernel<true>, gemm_resid_grid(g.pack_tiles, g.K), 256, 0, stream, g);
        return;
    }
    if (g.M <= kStreamMaxRows && g.wpack && g.x_resid) {
        ScopedProf sp(PSD_KIND_GEMM_COLUMN, stream);
        const int grid = g.N / 16;                        // every segment is a multiple of 64 wide; M <= 16: one row tile
        launch_kernel(gemm_bf16_column_kernel<1, 16>, grid, 1024, 0, stream, g);
        return;
    }
    // the unit kernel addresses the activation rows with 32-bit offsets from the first one
    const bool x_near = (long)(x_row(g, g.M - 1) - x_row(g, 0) + 1) * g.K * 4 < 0x7fff0000L;
    if (g.M <= kStreamMaxRows && g.wpack && x_near) {
        ScopedProf sp(PSD_KIND_GEMM_SKINNY, stream);
        launch_kernel(gemm_bf16_unit_kernel<false>, gemm_stream_grid(g.pack_tiles, g.K), 256, 0, stream, g);
    } else if (g.M <= kStreamMaxRows) {
        ScopedProf sp(PSD_KIND_GEMM_SLOT, stream);
        dim3 grid(tiles_of(g.n, g.nseg, kSkinnyRows), g.splitk);
        launch_kernel(gemm_bf16_skinny_kernel<1>, grid, 256, 0, stream, g);
    } else {
        ScopedProf sp(PSD_KIND_GEMM_TILED, stream);
        int nb, sk;
        tiled_choice(g.M, g.K, g.n, g.nseg, &nb, &sk);
        if (sk != g.splitk) nb = 6;                       // the caller sized the partial slots for its own split
        const int bm = tiled_block_rows(g.M);
        dim3 grid(tiles_of(g.n, g.nseg, 32 * nb) * ((g.M + bm - 1) / bm), g.splitk);
        auto go = [&](auto kernel) {
            // opt in to more than 64 KB of dynamic LDS: a property of the function on the current device, set before
            // every launch (a cheap host call) so that no process-wide flag has to remember who set it where
            const size_t lds = (size_t)(bm + 32 * nb) * kLdsStride * sizeof(uint16_t) * (bm == 256 ? 2 : 1);
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)lds);
            launch_kernel(kernel, grid, bm * 2, lds, stream, g);
        };
        if (g.w4 && bm == 256) {
            if (nb == 4) go(gemm_f16_tiled_kernel<4, 4, true>);
            else if (nb == 6) go(gemm_f16_tiled_kernel<6, 4, true>);
            else go(gemm_f16_tiled_kernel<8, 4, true>);
        } else if (g.w4) {
            if (nb == 4) go(gemm_f16_tiled_kernel<4, 2, true>);
            else if (nb == 6) go(gemm_f16_tiled_kernel<6, 2, true>);
            else go(gemm_f16_tiled_kernel<8, 2, true>);
        } else if (bm == 256) {
            if (nb == 4) go(gemm_f16_tiled_kernel<4, 4>);
            else if (nb == 6) go(gemm_f16_tiled_kernel<6, 4>);
            else go(gemm_f16_tiled_kernel<8, 4>);
        } else {
            if (nb == 4) go(gemm_f16_tiled_kernel<4, 2>);
            else if (nb == 6) go(gemm_f16_tiled_kernel<6, 2>);
            else go(gemm_f16_tiled_kernel<8, 2>);
        }
    }
    if (g.reduced) {
        const dim3 grid((unsigned)((g.N + 255) / 256), (unsigned)g.M);
        ScopedProf sp(PSD_KIND_GEMM_REDUCE, stream);
        launch_kernel(gemm_splitk_reduce_kernel, grid, 256, 0, stream, g);
    }
}

}  // namespace psd
