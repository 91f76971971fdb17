// Calibration kernels: what this chip sustains on the access and issue patterns the hot path is made of,
// measured through the same library the benchmark times (a plain stream read, a copy, a gather of KV rows
// in the attention kernels' access shape, and back-to-back matrix instructions).  Measurement aids, not
// part of the computation.
#include "ic_common.hpp"

namespace ic {

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;

// Every thread reads 16-byte vectors, grid-strided, and folds them; one word per workgroup leaves the chip.
__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4 *src, int64_t n_vec, uint32_t *out)
{
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * 256 * 4;
    for (int64_t i = (int64_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n_vec; i += stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = (i + 256 * u < n_vec) ? src[i + 256 * u] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;          // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void calib_copy_kernel(const u32x4 *src, u32x4 *dst, int64_t n_vec)
{
    const int64_t stride = (int64_t)gridDim.x * 256 * 4;
    for (int64_t i = (int64_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n_vec; i += stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = (i + 256 * u < n_vec) ? src[i + 256 * u] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + 256 * u < n_vec) dst[i + 256 * u] = v[u];
    }
}

// Gather of whole rows of `row_bytes` (a multiple of 128): eight lanes fetch one 128-byte line, a wave 8 rows
// per round, every load of a row group in flight before any is consumed.  idx entries are clamped to the table.
template <int LINES>
__global__ __launch_bounds__(256) void calib_gather_kernel(const unsigned char *src, const int32_t *idx, int64_t n_rows,
                                                           int64_t table_rows, uint32_t *out)
{
    const int lane = threadIdx.x & 63, gr = lane >> 3, gp = lane & 7;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (int64_t)gridDim.x * 4;
    uint32_t acc = 0;
    for (int64_t r0 = wave * 8; r0 < n_rows; r0 += n_waves * 8) {
        const int64_t r = r0 + gr;
        int64_t row = r < n_rows ? idx[r] : 0;
        row = row < 0 ? 0 : (row >= table_rows ? table_rows - 1 : row);
        const u32x4 *p = (const u32x4 *)(src + row * (int64_t)(LINES * 128)) + gp;
        u32x4 v[LINES];
#pragma unroll
        for (int l = 0; l < LINES; ++l) v[l] = p[8 * l];
#pragma unroll
        for (int l = 0; l < LINES; ++l) acc ^= v[l][0] ^ v[l][1] ^ v[l][2] ^ v[l][3];
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;
}

// Back-to-back matrix instructions on four independent accumulators per wave (no memory traffic).
template <bool FP8>
__global__ __launch_bounds__(256) void calib_mfma_kernel(int iters, float *out)
{
    f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    const int lane = threadIdx.x & 63;
    if constexpr (FP8) {
        i32x8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[i] = 0x38383838 + lane;                      // e4m3 bytes near 1.0
            b[i] = 0x30303030 + i;
        }
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[c], 0, 0, 0, 0, 0, 0);
    } else {
        bf16x8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[i] = (__bf16)(0.001f * (lane + i));
            b[i] = (__bf16)(0.002f * (lane - i));
        }
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[c][i];
    if (s == 12345.678f) out[blockIdx.x * 256 + threadIdx.x] = s;
}

// The data movement of the prefill attention kernel's tile loop without its arithmetic: tiles of 64 table rows of
// 1152 bytes, four waves, wave w rows 16 w .. 16 w + 15.  PARTS: 1 = gather into registers only (18 loads per lane
// and tile, eight lanes per 128-byte line, one tile ahead); 2 = + store the tile to LDS (row-major, rows padded by 32 bytes, double
// buffered, one barrier per tile); 3 = + read it back as an A operand would be (16-byte reads, once per byte);
// 4 = + read its first 1024 bytes per row through the transposing 8-byte read, once per byte.  Everything read is
// folded into one word so that nothing is dropped.
template <int PARTS>
__global__ __launch_bounds__(256, 1) void calib_tilepath_kernel(const unsigned char *src, const int32_t *idx, int64_t n_rows,
                                                                int64_t table_rows, uint32_t *out)
{
    constexpr int ROWG = 1152, ROWB = ROWG + 32, KS = 18, TBUFB = 64 * ROWB;   // row in memory, row stride in LDS
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][64][ROWB]
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4, hh = lane >> 5;
    const int gr = lane >> 3, gp = lane & 7;
    const int st_off = (16 * wave + gr) * ROWB + (gp << 4);
    const int ka_row = (16 * wave + l16) * ROWB;
    const int ka_e = ka_row + (g << 4), ka_o = ka_row + ((4 + g) << 4);
    const int tr_row = 8 * hh + 2 * (l16 >> 2);           // the four rows of a transpose read are two apart
    const int tr_slot = 4 * (wave & 1) + 2 * (g & 1) + ((l16 & 3) >> 1);
    const int tr0 = tr_row * ROWB + 128 * (wave >> 1) + (tr_slot << 4) + 8 * (l16 & 1);
    const int tr1 = tr0 + ROWB;
    const int64_t n_tiles = n_rows / 64;
    // the row numbers of a tile are requested a tile before its rows are (as the attention kernel does), so that
    // no gather waits for them
    auto row_id = [&](int64_t tile, int half) {
        const int64_t r = (tile < n_tiles ? tile : n_tiles - 1) * 64 + 16 * wave + 8 * half + gr;
        return idx[r];
    };
    auto row_ptr = [&](int32_t id) {
        const int64_t row = id < 0 ? 0 : (id >= table_rows ? table_rows - 1 : (int64_t)id);
        return (const u32x4 *)(src + row * ROWG) + gp;
    };
    u32x4 cur[KS];
    uint32_t acc = 0;
    int64_t t = blockIdx.x;
    if (t >= n_tiles) return;
    {
        const u32x4 *pl = row_ptr(row_id(t, 0)), *ph = row_ptr(row_id(t, 1));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cur[ks] = ((ks & 1) ? ph : pl)[8 * (ks >> 1)];
    }
    int32_t id_lo = row_id(t + gridDim.x, 0), id_hi = row_id(t + gridDim.x, 1);
    int buf = 0;
    for (; t < n_tiles; t += gridDim.x, buf ^= 1) {
        unsigned char *tb = smem + buf * TBUFB;
        const u32x4 *pl = row_ptr(id_lo), *ph = row_ptr(id_hi);
        id_lo = row_id(t + 2 * (int64_t)gridDim.x, 0);
        id_hi = row_id(t + 2 * (int64_t)gridDim.x, 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if constexpr (PARTS >= 2)
                *(u32x4 *)(tb + st_off + (ks & 1) * 8 * ROWB + 128 * (ks >> 1)) = cur[ks];
            else
                acc ^= cur[ks][0] ^ cur[ks][1] ^ cur[ks][2] ^ cur[ks][3];
            cur[ks] = ((ks & 1) ? ph : pl)[8 * (ks >> 1)];
        }
        if constexpr (PARTS >= 2) __syncthreads();
        // (the reads of a phase are all issued before the first of them is looked at, as a kernel that feeds them
        // to the matrix pipes through a ring of registers would have them in flight)
        if constexpr (PARTS >= 3) {
            u32x4 v[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) v[ks] = *(const u32x4 *)(tb + ((ks & 1) ? ka_o : ka_e) + 128 * (ks >> 1));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc ^= v[ks][0] ^ v[ks][1] ^ v[ks][2] ^ v[ks][3];
        }
        if constexpr (PARTS >= 4) {
#pragma unroll
            for (int jh = 0; jh < 2; ++jh) {
                s16x4 va[2][4], vb[2][4];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        const int j = 2 * jh + jj;
                        va[jj][nb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tb + tr0 + 16 * j * ROWB + 256 * nb));
                        vb[jj][nb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tb + tr1 + 16 * j * ROWB + 256 * nb));
                    }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        const s16x4 a = va[jj][nb], b = vb[jj][nb];
                        acc ^= (uint32_t)(uint16_t)(a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3]);
                    }
            }
        }
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;
}

// The same bytes per tile as calib_tilepath_kernel<4>, moved by eight waves (two per SIMD) instead of four: wave w
// gathers and stores rows 8 w .. + 7, reads the score operand of rows 16 (w & 3) .. + 15 for the contraction steps
// of parity w >> 2, and does the transpose reads of column block w & 3 for the row groups 2 (w >> 2), + 1.  No byte
// is read twice.  (An attention kernel cannot be laid out this way as it stands: a wave that computes scores for
// all heads holds all of Q, 144 registers, and at two waves per SIMD a wave has 256.)
__global__ __launch_bounds__(512, 1) void calib_tilepath8_kernel(const unsigned char *src, const int32_t *idx, int64_t n_rows,
                                                                 int64_t table_rows, uint32_t *out)
{
    constexpr int ROWG = 1152, ROWB = ROWG + 32, LINES = 9, TBUFB = 64 * ROWB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][64][ROWB]
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4, hh = lane >> 5;
    const int gr = lane >> 3, gp = lane & 7;
    const int cb = wave & 3, par = wave >> 2;
    const int st_off = (8 * wave + gr) * ROWB + (gp << 4);
    const int ka_row = (16 * cb + l16) * ROWB;
    const int ka_e = ka_row + (g << 4), ka_o = ka_row + ((4 + g) << 4);
    const int tr_row = 8 * hh + 2 * (l16 >> 2);           // the four rows of a transpose read are two apart
    const int tr_slot = 4 * (cb & 1) + 2 * (g & 1) + ((l16 & 3) >> 1);
    const int tr0 = tr_row * ROWB + 128 * (cb >> 1) + (tr_slot << 4) + 8 * (l16 & 1);
    const int tr1 = tr0 + ROWB;
    const int64_t n_tiles = n_rows / 64;
    auto row_id = [&](int64_t tile) {
        const int64_t r = (tile < n_tiles ? tile : n_tiles - 1) * 64 + 8 * wave + gr;
        return idx[r];
    };
    auto row_ptr = [&](int32_t id) {
        const int64_t row = id < 0 ? 0 : (id >= table_rows ? table_rows - 1 : (int64_t)id);
        return (const u32x4 *)(src + row * ROWG) + gp;
    };
    u32x4 cur[LINES];
    uint32_t acc = 0;
    int64_t t = blockIdx.x;
    if (t >= n_tiles) return;
    {
        const u32x4 *pr = row_ptr(row_id(t));
#pragma unroll
        for (int c = 0; c < LINES; ++c) cur[c] = pr[8 * c];
    }
    int32_t id_n = row_id(t + gridDim.x);
    int buf = 0;
    for (; t < n_tiles; t += gridDim.x, buf ^= 1) {
        unsigned char *tb = smem + buf * TBUFB;
        const u32x4 *pr = row_ptr(id_n);
        id_n = row_id(t + 2 * (int64_t)gridDim.x);
#pragma unroll
        for (int c = 0; c < LINES; ++c) {
            *(u32x4 *)(tb + st_off + 128 * c) = cur[c];
            cur[c] = pr[8 * c];
        }
        __syncthreads();
        {
            u32x4 v[LINES];
#pragma unroll
            for (int i = 0; i < LINES; ++i) {
                const int ks = 2 * i + par;
                v[i] = *(const u32x4 *)(tb + (par ? ka_o : ka_e) + 128 * (ks >> 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < LINES; ++i) acc ^= v[i][0] ^ v[i][1] ^ v[i][2] ^ v[i][3];
        }
        {
            s16x4 va[2][4], vb[2][4];
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const int j = 2 * par + jj;
                    va[jj][nb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tb + tr0 + 16 * j * ROWB + 256 * nb));
                    vb[jj][nb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tb + tr1 + 16 * j * ROWB + 256 * nb));
                }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const s16x4 a = va[jj][nb], b = vb[jj][nb];
                    acc ^= (uint32_t)(uint16_t)(a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3]);
                }
        }
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;
}

// The four-wave movement of calib_tilepath_kernel<4> with its phases merged: the 18 store + gather pairs that stage
// tile t + 1 and fetch tile t + 2 are spread evenly between the 50 reads of tile t (two buffers, one barrier per
// tile, row numbers three tiles ahead), so that the vector memory queue and the LDS pipe work at the same time.
__global__ __launch_bounds__(256, 1) void calib_tilepath_il_kernel(const unsigned char *src, const int32_t *idx, int64_t n_rows,
                                                                   int64_t table_rows, uint32_t *out)
{
    constexpr int ROWG = 1152, ROWB = ROWG + 32, KS = 18, TBUFB = 64 * ROWB;   // row in memory, row stride in LDS
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][64][ROWB]
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4, hh = lane >> 5;
    const int gr = lane >> 3, gp = lane & 7;
    const int st_off = (16 * wave + gr) * ROWB + (gp << 4);
    const int ka_row = (16 * wave + l16) * ROWB;
    const int ka_e = ka_row + (g << 4), ka_o = ka_row + ((4 + g) << 4);
    const int tr_row = 8 * hh + 2 * (l16 >> 2);           // the four rows of a transpose read are two apart
    const int tr_slot = 4 * (wave & 1) + 2 * (g & 1) + ((l16 & 3) >> 1);
    const int tr0 = tr_row * ROWB + 128 * (wave >> 1) + (tr_slot << 4) + 8 * (l16 & 1);
    const int tr1 = tr0 + ROWB;
    const int64_t n_tiles = n_rows / 64;
    auto row_id = [&](int64_t tile, int half) {
        const int64_t r = (tile < n_tiles ? tile : n_tiles - 1) * 64 + 16 * wave + 8 * half + gr;
        return idx[r];
    };
    auto row_ptr = [&](int32_t id) {
        const int64_t row = id < 0 ? 0 : (id >= table_rows ? table_rows - 1 : (int64_t)id);
        return (const u32x4 *)(src + row * ROWG) + gp;
    };
    u32x4 cur[KS];
    uint32_t acc = 0;
    int64_t t = blockIdx.x;
    if (t >= n_tiles) return;
    const int64_t G = gridDim.x;
    {
        const u32x4 *pl = row_ptr(row_id(t, 0)), *ph = row_ptr(row_id(t, 1));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cur[ks] = ((ks & 1) ? ph : pl)[8 * (ks >> 1)];
        const u32x4 *ql = row_ptr(row_id(t + G, 0)), *qh = row_ptr(row_id(t + G, 1));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            *(u32x4 *)(smem + st_off + (ks & 1) * 8 * ROWB + 128 * (ks >> 1)) = cur[ks];
            cur[ks] = ((ks & 1) ? qh : ql)[8 * (ks >> 1)];
        }
    }
    int32_t id_lo = row_id(t + 2 * G, 0), id_hi = row_id(t + 2 * G, 1);
    __syncthreads();
    int buf = 0;
    for (; t < n_tiles; t += G, buf ^= 1) {
        const unsigned char *tb = smem + buf * TBUFB;      // tile t
        unsigned char *tn = smem + (buf ^ 1) * TBUFB;      // tile t + G goes here
        const u32x4 *pl = row_ptr(id_lo), *ph = row_ptr(id_hi);
        id_lo = row_id(t + 3 * G, 0);
        id_hi = row_id(t + 3 * G, 1);
        // 50 reads (18 of the score operand, 32 transposing ones) with the 18 store + gather pairs spread evenly
        // between them
        u32x4 v[KS];
        s16x4 va[4][4], vb[4][4];
        auto pair = [&](int ks) {
            *(u32x4 *)(tn + st_off + (ks & 1) * 8 * ROWB + 128 * (ks >> 1)) = cur[ks];
            cur[ks] = ((ks & 1) ? ph : pl)[8 * (ks >> 1)];
        };
#pragma unroll
        for (int r = 0; r < 50; ++r) {
            if (r < KS) {
                v[r] = *(const u32x4 *)(tb + ((r & 1) ? ka_o : ka_e) + 128 * (r >> 1));
            } else {
                const int e = r - KS, j = e >> 3, nb = (e >> 1) & 3;
                if (e & 1)
                    vb[j][nb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tb + tr1 + 16 * j * ROWB + 256 * nb));
                else
                    va[j][nb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tb + tr0 + 16 * j * ROWB + 256 * nb));
            }
            // pair k goes after read number floor((k + 1) * 50 / 18) - 1
            if ((r + 1) * KS / 50 != r * KS / 50) pair(r * KS / 50);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc ^= v[ks][0] ^ v[ks][1] ^ v[ks][2] ^ v[ks][3];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const s16x4 x = va[j][nb], y = vb[j][nb];
                acc ^= (uint32_t)(uint16_t)(x[0] ^ x[1] ^ x[2] ^ x[3] ^ y[0] ^ y[1] ^ y[2] ^ y[3]);
            }
        __syncthreads();
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;
}

// LDS access patterns of the attention tile by themselves: 16 waves per workgroup (one workgroup per CU keeps the
// LDS unit busy from every SIMD) issue `rounds` x 16 reads of one kind and fold what they read.  PATTERN 0: the
// 16-byte score-operand read (lane = row within 16, 16-byte piece lane / 16) with rows 1184 bytes apart, no
// swizzle; 1: the same read with rows 1152 bytes apart and the 16-byte slot XOR-swizzled by the row number; 2: the
// 8-byte transposing read over four rows TWO apart, rows 1184 apart; 3: the same over four consecutive rows.
template <int PATTERN>
__global__ __launch_bounds__(1024, 1) void calib_lds_kernel(int rounds, uint32_t *out)
{
    constexpr int kBytes = 96 * 1024;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < kBytes / 4; i += 1024) ((uint32_t *)smem)[i] = (uint32_t)i * 2654435761u;
    __syncthreads();
    const int l16 = lane & 15, g = lane >> 4, hh = lane >> 5;
    int off;
    if (PATTERN == 0) {
        off = l16 * 1184 + (g << 4);
    } else if (PATTERN == 1) {
        off = l16 * 1152 + ((g ^ (((l16 & 3) << 1) | ((l16 >> 2) & 1))) << 4);
    } else {
        const int row = 8 * hh + (PATTERN == 2 ? 2 : 1) * (l16 >> 2);
        off = row * 1184 + ((2 * (g & 1) + ((l16 & 3) >> 1)) << 4) + 8 * (l16 & 1);
    }
    typedef __attribute__((address_space(3))) unsigned char lds_u8;
    const lds_u8 *p = (const lds_u8 *)smem + off;         // + 15 * 4608 + 16 stays below kBytes for every pattern
    uint32_t acc = 0;
    for (int r = 0; r < rounds; ++r) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const lds_u8 *q = p + u * 4608;               // four rows of 1152 further: the same banks
            if (PATTERN <= 1) {
                const u32x4 v = *(const volatile __attribute__((address_space(3))) u32x4 *)q;
                acc ^= v[0] ^ v[3];
            } else {
                const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)q);
                acc ^= (uint32_t)(uint16_t)v[0] ^ (uint32_t)(uint16_t)v[3];
                asm volatile("" ::"v"(v));
            }
        }
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;
}

template <int PATTERN>
hipError_t launch_lds(void *dst, int64_t rounds, int wgs, hipStream_t st)
{
    constexpr int lds = 96 * 1024;
    static hipError_t attr = hipFuncSetAttribute((const void *)calib_lds_kernel<PATTERN>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((calib_lds_kernel<PATTERN>), dim3((unsigned)wgs), dim3(1024), lds, st, (int)rounds, (uint32_t *)dst);
    return hipGetLastError();
}

template <int PARTS>
hipError_t launch_tilepath(const void *src, void *dst, const int32_t *idx, int64_t n, int64_t table_rows, int wgs, hipStream_t st)
{
    constexpr int lds = 2 * 64 * (1152 + 32);
    static hipError_t attr = hipFuncSetAttribute((const void *)calib_tilepath_kernel<PARTS>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((calib_tilepath_kernel<PARTS>), dim3((unsigned)wgs), dim3(256), lds, st, (const unsigned char *)src, idx, n, table_rows,
                       (uint32_t *)dst);
    return hipGetLastError();
}

} // namespace

hipError_t launch_calib(int kind, const void *src, void *dst, const int32_t *idx, int64_t n, int64_t table_rows, int row_bytes,
                        int wgs, hipStream_t st)
{
    dim3 grid((unsigned)wgs), block(256);
    switch (kind) {
    case IC_CALIB_READ:
        hipLaunchKernelGGL(calib_read_kernel, grid, block, 0, st, (const u32x4 *)src, n / 16, (uint32_t *)dst);
        break;
    case IC_CALIB_COPY:
        hipLaunchKernelGGL(calib_copy_kernel, grid, block, 0, st, (const u32x4 *)src, (u32x4 *)dst, n / 16);
        break;
    case IC_CALIB_GATHER:
        if (row_bytes == 1152)
            hipLaunchKernelGGL((calib_gather_kernel<9>), grid, block, 0, st, (const unsigned char *)src, idx, n, table_rows, (uint32_t *)dst);
        else if (row_bytes == 256)
            hipLaunchKernelGGL((calib_gather_kernel<2>), grid, block, 0, st, (const unsigned char *)src, idx, n, table_rows, (uint32_t *)dst);
        else
            return hipErrorInvalidValue;
        break;
    case IC_CALIB_MFMA_BF16:
        hipLaunchKernelGGL((calib_mfma_kernel<false>), grid, block, 0, st, (int)n, (float *)dst);
        break;
    case IC_CALIB_MFMA_FP8:
        hipLaunchKernelGGL((calib_mfma_kernel<true>), grid, block, 0, st, (int)n, (float *)dst);
        break;
    case IC_CALIB_TILE_GATHER:
        return launch_tilepath<1>(src, dst, idx, n, table_rows, wgs, st);
    case IC_CALIB_TILE_STORE:
        return launch_tilepath<2>(src, dst, idx, n, table_rows, wgs, st);
    case IC_CALIB_TILE_READ:
        return launch_tilepath<3>(src, dst, idx, n, table_rows, wgs, st);
    case IC_CALIB_TILE_READ2:
        return launch_tilepath<4>(src, dst, idx, n, table_rows, wgs, st);
    case IC_CALIB_TILE_INTERLEAVED: {
        constexpr int lds = 2 * 64 * (1152 + 32);
        static hipError_t attr = hipFuncSetAttribute((const void *)calib_tilepath_il_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(calib_tilepath_il_kernel, grid, dim3(256), lds, st, (const unsigned char *)src, idx, n, table_rows, (uint32_t *)dst);
        break;
    }
    case IC_CALIB_TILE_8WAVES: {
        constexpr int lds = 2 * 64 * (1152 + 32);
        static hipError_t attr = hipFuncSetAttribute((const void *)calib_tilepath8_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(calib_tilepath8_kernel, grid, dim3(512), lds, st, (const unsigned char *)src, idx, n, table_rows, (uint32_t *)dst);
        break;
    }
    case IC_CALIB_LDS_READ16_PADDED:
        return launch_lds<0>(dst, n, wgs, st);
    case IC_CALIB_LDS_READ16_SWIZZLED:
        return launch_lds<1>(dst, n, wgs, st);
    case IC_CALIB_LDS_TR8_ROWS2:
        return launch_lds<2>(dst, n, wgs, st);
    case IC_CALIB_LDS_TR8_ROWS1:
        return launch_lds<3>(dst, n, wgs, st);
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace ic
