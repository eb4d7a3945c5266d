// gfx950 kernels of the verification pass.
//
// One persistent kernel runs a whole segment of the pass (embedding, a range of
// layers, optionally an LM head with its accept step) as a list of phases with
// a grid-wide barrier between consecutive phases.  "P" phases stream weights or
// the KV cache (HBM-bound), "R" phases reduce partial results and apply the
// element-wise epilogues (latency-bound, tiny).
//
// Per layer (Eq. 3 of the paper, f = Llama-2 block):
//   P_QKV  x_hat . [Wq;Wk;Wv]^T                       -> partials
//   R_QKV  reduce, * rstd, RoPE, q -> scratch, k/v -> paged bf16 cache
//   P_ATT  causal attention of the new rows over the cache, split over positions
//   R_ATT  merge the splits                            -> attn
//   P_O    attn . Wo^T                                 -> partials
//   R_O    h += ., sum of squares, x_hat = g_ffn * h   -> xn
//   P_GU   x_hat . [Wg;Wu]^T                           -> partials
//   R_GU   silu(rstd*gate) * (rstd*up)                 -> u
//   P_DN   u . Wd^T                                    -> partials
//   R_DN   h += ., sum of squares, x_hat for the next layer and/or the head
// Head (z^(l) = LMHead(h^(l)); accept rule of Eq. 2 / Eq. 5):
//   P_HEAD x_hat . W_lm^T -> partials; R_HEAD reduce, * rstd, per-workgroup
//   argmax; R_ACCEPT global argmax (lowest id wins ties), accept length,
//   publication to pinned host memory, KV commit.
//
// RMSNorm is split: the GEMM input is g * h; the row factor
// rstd = 1/sqrt(mean(h^2)+eps) is applied to the fp32 GEMM result, which is
// the same product because rstd is constant along K.
#pragma once

#include "ee_device.hpp"

namespace ee {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// 16-byte streaming load (weights are read once per pass: no reuse in cache)
__device__ __forceinline__ uint4 load_stream16(const uint4 *p)
{
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even; inputs are finite
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void unpack8(const uint4 &v, float *f)
{
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xFFFF0000u);
    f[4] = __uint_as_float(v.z << 16);
    f[5] = __uint_as_float(v.z & 0xFFFF0000u);
    f[6] = __uint_as_float(v.w << 16);
    f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

// ------------------------------------------------------------------ grid barrier

// Sense-reversing barrier over all workgroups of a cooperative launch.  The
// wait is bounded: after spin_limit polls the workgroup raises *err and goes
// on, and every later barrier falls through, so the grid always drains.
__device__ __forceinline__ void grid_barrier(GridBarrier *b, unsigned nwg, int *err, unsigned spin_limit)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned gen = __hip_atomic_load(&b->gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        unsigned prev = __hip_atomic_fetch_add(&b->count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev == nwg - 1) {
            __hip_atomic_store(&b->count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&b->gen, gen + 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            unsigned spins = 0;
            while (__hip_atomic_load(&b->gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gen) {
                if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                if (++spins > spin_limit) {
                    __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

// ------------------------------------------------------------------ rows

__device__ __forceinline__ int row_pos(const PassArgs &a, int r)
{
    if (a.mode == 1) return a.pf_pos0 + r;
    int s = r / a.M;
    return a.sess[s].state[0] + (r - s * a.M);
}

__device__ __forceinline__ int row_token(const PassArgs &a, int r)
{
    if (a.mode == 1) return a.pf_tokens[r];
    int s = r / a.M, i = r - s * a.M;
    return i == 0 ? a.sess[s].state[1] : a.sess[s].drafts[i - 1];
}

// rstd[m] = 1/sqrt(sum_g ss[g][m] / d + eps) into LDS, fixed summation order
__device__ __forceinline__ void load_rstd(const float *ss, int nwg, int rows_max, int rows, int d, float eps,
                                          float *rstd_lds)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int m = wave; m < rows; m += WAVES_PER_WG) {
        float s = 0.f;
        for (int g = lane; g < nwg; g += 64) s += ss[(size_t)g * rows_max + m];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) rstd_lds[m] = 1.0f / sqrtf(s / (float)d + eps);
    }
    __syncthreads();
}

// ------------------------------------------------------------------ tile index arithmetic

struct TilePos {
    int kb, nt, kti, klen;
};

__device__ __forceinline__ TilePos tile_decode(const GemmPlan &pl, long long t)
{
    TilePos p;
    const long long B = (long long)pl.NT * pl.KBT;
    const long long full = (long long)(pl.nKB - 1) * B;
    if (t < full) {
        p.kb = (int)(t / B);
        int rem = (int)(t - (long long)p.kb * B);
        p.nt = rem / pl.KBT;
        p.kti = rem - p.nt * pl.KBT;
        p.klen = pl.KBT;
    } else {
        p.kb = pl.nKB - 1;
        int rem = (int)(t - full);
        p.nt = rem / pl.KBT_last;
        p.kti = rem - p.nt * pl.KBT_last;
        p.klen = pl.KBT_last;
    }
    return p;
}

// wave that streams tile t: the w with floor(T*w/NW) <= t < floor(T*(w+1)/NW)
__device__ __forceinline__ int tile_owner(long long T, int NW, long long t)
{
    return (int)(((t + 1) * (long long)NW - 1) / T);
}

// ------------------------------------------------------------------ P: weight-streaming GEMM

// partial[run][piece][m][16] = W_tile(16 x 32) . x_hat^T(32 x rows) summed over the tiles of
// the run that fall into this wave's range.  x: fp32 [rows][ldx], already scaled by the norm
// gain.  The MFMA takes bf16 operands; x is fed as two bf16 terms, hi = bf16(x) and
// lo = bf16(x - hi), so that the activations keep about 16 mantissa bits (the weights are
// exact bf16 values).  The matrix cores are idle most of the time in this HBM-bound loop,
// so the second MFMA per tile is free.
template <int MT>
__device__ void gemm_phase(const GemmPlan &pl, const uint4 *__restrict__ W, const float *__restrict__ x,
                           int ldx, int rows, int rows_max, int nwg, char *lds)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int NW = nwg * WAVES_PER_WG;
    const long long T = pl.T;
    const int w0 = blockIdx.x * WAVES_PER_WG;
    const long long g0 = T * w0 / NW, g1 = T * (w0 + WAVES_PER_WG) / NW;
    if (g0 >= g1) return;  // uniform over the workgroup

    const int kb_lo = tile_decode(pl, g0).kb, kb_hi = tile_decode(pl, g1 - 1).kb;
    const int xs_stride = pl.KBT * 32 + 8;                  // bf16 elements per staged row
    uint16_t *xs_hi = reinterpret_cast<uint16_t *>(lds);    // [rows][xs_stride]
    uint16_t *xs_lo = xs_hi + (size_t)rows * xs_stride;
    const long long t0 = T * (w0 + wave) / NW, t1 = T * (w0 + wave + 1) / NW;
    const long long B = (long long)pl.NT * pl.KBT;

    int brow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) brow[mt] = min(mt * 16 + (lane & 15), rows - 1) * xs_stride;
    const int bk = (lane >> 4) * 8;
    const size_t pstride = (size_t)rows_max * 16;
    constexpr int D = 8;  // tiles in flight per wave (8 KB)

    for (int kb = kb_lo; kb <= kb_hi; ++kb) {
        if (kb > kb_lo) __syncthreads();
        // stage K-block kb of x_hat as hi/lo bf16
        {
            const int c8_per_row = pl.KBT * 4;  // 8-element chunks per row
            const int total = rows * c8_per_row;
            for (int i = tid; i < total; i += WG_THREADS) {
                int row = i / c8_per_row, c = i - row * c8_per_row;
                int k = kb * pl.KBT * 32 + c * 8;
                uint4 hi = make_uint4(0, 0, 0, 0), lo = make_uint4(0, 0, 0, 0);
                if (k < ldx) {
                    const float4 *src = reinterpret_cast<const float4 *>(x + (size_t)row * ldx + k);
                    float4 a = src[0], b = src[1];
                    float f[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                    uint32_t h[8], l[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        h[e] = f32_to_bf16(f[e]);
                        l[e] = f32_to_bf16(f[e] - bf16_to_f32((uint16_t)h[e]));
                    }
                    hi = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
                    lo = make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16));
                }
                *reinterpret_cast<uint4 *>(xs_hi + (size_t)row * xs_stride + c * 8) = hi;
                *reinterpret_cast<uint4 *>(xs_lo + (size_t)row * xs_stride + c * 8) = lo;
            }
        }
        __syncthreads();

        // this wave's tiles inside K-block kb
        const int klen = (kb == pl.nKB - 1) ? pl.KBT_last : pl.KBT;
        const long long blk_start = (long long)kb * B, blk_end = blk_start + (long long)pl.NT * klen;
        const long long ta = t0 > blk_start ? t0 : blk_start, tb = t1 < blk_end ? t1 : blk_end;
        if (ta >= tb) continue;
        const int n = (int)(tb - ta);
        int rem = (int)(ta - blk_start);
        int nt = rem / klen, kti = rem - nt * klen;
        // the first run may have been begun by earlier waves
        int piece = (w0 + wave) - tile_owner(T, NW, blk_start + (long long)nt * klen);

        f32x4_t acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

        const uint4 *wp = W + (size_t)ta * 64 + lane;
        uint4 buf[D];
#pragma unroll
        for (int j = 0; j < D; ++j)
            if (j < n) buf[j] = load_stream16(wp + (size_t)j * 64);

        for (int i = 0; i < n; i += D) {
#pragma unroll
            for (int j = 0; j < D; ++j) {
                if (i + j < n) {
                    uint4 av = buf[j];
                    if (i + j + D < n) buf[j] = load_stream16(wp + (size_t)(i + j + D) * 64);
                    bf16x8_t A = __builtin_bit_cast(bf16x8_t, av);
                    const int xo = kti * 32 + bk;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        uint4 bh = *reinterpret_cast<const uint4 *>(xs_hi + brow[mt] + xo);
                        uint4 bl = *reinterpret_cast<const uint4 *>(xs_lo + brow[mt] + xo);
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8_t, bh), acc[mt], 0, 0, 0);
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8_t, bl), acc[mt], 0, 0, 0);
                    }
                    ++kti;
                    if (kti == klen || i + j + 1 == n) {
                        // D layout: lane holds rows (lane>>4)*4 .. +3 of N, column (lane&15) of M
                        float *dst = pl.part + ((size_t)(kb * pl.NT + nt) * pl.MAXP + piece) * pstride;
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            int m = mt * 16 + (lane & 15);
                            if (m < rows)
                                *reinterpret_cast<float4 *>(dst + (size_t)m * 16 + (lane >> 4) * 4) =
                                    make_float4(acc[mt][0], acc[mt][1], acc[mt][2], acc[mt][3]);
                            acc[mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                        }
                        piece = 0;
                        if (kti == klen) {
                            kti = 0;
                            ++nt;
                        }
                    }
                }
            }
        }
    }
}

__device__ __forceinline__ void gemm_dispatch(const GemmPlan &pl, const uint4 *W, const float *x, int ldx,
                                              int rows, int rows_max, int nwg, char *lds)
{
    if (rows <= 16)
        gemm_phase<1>(pl, W, x, ldx, rows, rows_max, nwg, lds);
    else if (rows <= 32)
        gemm_phase<2>(pl, W, x, ldx, rows, rows_max, nwg, lds);
    else
        gemm_phase<3>(pl, W, x, ldx, rows, rows_max, nwg, lds);
}

// sum of all partials of output (m, n), fixed order (K-block, then piece)
__device__ __forceinline__ float reduce_out(const GemmPlan &pl, int rows_max, int m, int n)
{
    const size_t pstride = (size_t)rows_max * 16;
    const float *p = pl.part + ((size_t)(n >> 4) * pl.MAXP) * pstride + (size_t)m * 16 + (n & 15);
    const size_t kb_stride = (size_t)pl.NT * pl.MAXP * pstride;
    float s = 0.f;
    for (int kb = 0; kb < pl.nKB; ++kb) {
        for (int pc = 0; pc < pl.MAXP; ++pc) s += p[(size_t)pc * pstride];
        p += kb_stride;
    }
    return s;
}

// ------------------------------------------------------------------ R: residual stream

// Columns [g*cw, (g+1)*cw) of every row belong to workgroup g.
//   SRC 0: h = embedding of the row's token (or the supplied embedding row)
//   SRC 1: h += reduced GEMM output of plan pl
// Then: partial sum of squares per row -> ss[g][m]; x_hat = gain * h (bf16) for
// up to two consumers (next layer's GEMM, LM head).
template <int SRC>
__device__ void resid_phase(const PassArgs &a, const GemmPlan *pl, const float *gain1, float *x1,
                            const float *gain2, float *x2, float *ss, char *lds)
{
    const ModelDev &md = *a.md;
    const int d = md.d, rows = a.rows, tid = threadIdx.x;
    const int cw = (d + a.nwg - 1) / a.nwg;
    const int n0 = blockIdx.x * cw;
    const int ncol = max(0, min(cw, d - n0));
    float *sq = reinterpret_cast<float *>(lds);  // [rows][cw]
    const int items = rows * ncol;
    for (int it = tid; it < items; it += WG_THREADS) {
        int m = it / ncol, c = it - m * ncol, n = n0 + c;
        float v;
        if (SRC == 0) {
            int tok = row_token(a, m);
            v = tok >= 0 ? bf16_to_f32(md.emb[(size_t)tok * d + n]) : bf16_to_f32(a.pf_emb[(size_t)m * d + n]);
        } else {
            v = a.sc.h[(size_t)m * d + n] + reduce_out(*pl, md.rows_max, m, n);
        }
        a.sc.h[(size_t)m * d + n] = v;
        sq[m * cw + c] = v * v;
        if (x1) x1[(size_t)m * md.Kpad_d + n] = gain1[n] * v;
        if (x2) x2[(size_t)m * md.Kpad_d + n] = gain2[n] * v;
    }
    __syncthreads();
    if (tid < rows) {
        float s = 0.f;
        for (int c = 0; c < ncol; ++c) s += sq[tid * cw + c];
        ss[(size_t)blockIdx.x * md.rows_max + tid] = s;
    }
}

// ------------------------------------------------------------------ R_QKV: reduce, RoPE, cache write

__device__ void rqkv_phase(const PassArgs &a, int layer, char *lds)
{
    const ModelDev &md = *a.md;
    const int d = md.d, hd = md.hd, half = hd >> 1, H = md.H, rows = a.rows;
    float *rstd = reinterpret_cast<float *>(lds);
    load_rstd(a.sc.ss_a, a.nwg, md.rows_max, rows, d, md.eps, rstd);
    const int per_row = 3 * (d >> 1);
    const int items = rows * per_row;
    const int gsz = a.nwg * WG_THREADS;
    for (int it = blockIdx.x * WG_THREADS + threadIdx.x; it < items; it += gsz) {
        int m = it / per_row, c = it - m * per_row;
        int sect = c / (d >> 1);       // 0 q, 1 k, 2 v
        int cc = c - sect * (d >> 1);
        int s = a.mode == 1 ? 0 : m / a.M;
        int pos = row_pos(a, m);
        const SessDev &sd = a.sess[s];
        float rs = rstd[m];
        if (sect < 2) {
            int head = cc / half, j = cc - head * half;
            int n0 = head * hd + j, n1 = n0 + half;
            float x0 = rs * reduce_out(md.qkv, md.rows_max, m, sect * d + n0);
            float x1 = rs * reduce_out(md.qkv, md.rows_max, m, sect * d + n1);
            float2 cs = sd.rope[(size_t)pos * half + j];
            float y0 = x0 * cs.x - x1 * cs.y;
            float y1 = x1 * cs.x + x0 * cs.y;
            if (sect == 0) {
                a.sc.q[(size_t)m * d + n0] = y0;
                a.sc.q[(size_t)m * d + n1] = y1;
            } else {
                int page = sd.page_table[pos / KV_PAGE];
                size_t base = ((((size_t)layer * sd.n_pages + page) * H + head) * KV_PAGE + (pos % KV_PAGE)) * hd;
                sd.kpool[base + j] = f32_to_bf16(y0);
                sd.kpool[base + j + half] = f32_to_bf16(y1);
            }
        } else {
            int n0 = cc * 2;
            int head = n0 / hd, e = n0 - head * hd;
            float v0 = rs * reduce_out(md.qkv, md.rows_max, m, 2 * d + n0);
            float v1 = rs * reduce_out(md.qkv, md.rows_max, m, 2 * d + n0 + 1);
            int page = sd.page_table[pos / KV_PAGE];
            size_t base = ((((size_t)layer * sd.n_pages + page) * H + head) * KV_PAGE + (pos % KV_PAGE)) * hd;
            uint32_t pk = (uint32_t)f32_to_bf16(v0) | ((uint32_t)f32_to_bf16(v1) << 16);
            *reinterpret_cast<uint32_t *>(sd.vpool + base + e) = pk;
        }
    }
}

// ------------------------------------------------------------------ P_ATT: split attention

constexpr float ATT_NEG = -1.0e30f;  // finite stand-in for "no position seen yet"

// Work item = (session, head, chunk of up to ATT_ROWS query rows, split of the
// position range).  Each wave takes a contiguous part of the split; a group of
// HD/8 lanes handles one cached position per step (16-byte loads of K and V).
// Output per item: un-normalised accumulator, running max and sum per row.
template <int HD>
__device__ void att_phase(const PassArgs &a, int layer, char *lds)
{
    constexpr int LPP = HD / 8;    // lanes per position
    constexpr int PPI = 64 / LPP;  // positions per wave step
    constexpr int REC = HD + 2;
    const ModelDev &md = *a.md;
    const int H = md.H, d = md.d, M = a.M;
    const int n_chunks = (M + ATT_ROWS - 1) / ATT_ROWS;
    const int n_splits = a.att_splits;
    const int n_items = a.n_sess * H * n_chunks * n_splits;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = lane / LPP, e8 = lane % LPP;
    float *wbuf = reinterpret_cast<float *>(lds);  // [WAVES][ATT_ROWS][REC]

    for (int item = blockIdx.x; item < n_items; item += a.nwg) {
        int unit = item / n_splits, sp = item - unit * n_splits;
        int s = unit / (H * n_chunks), rem = unit - s * (H * n_chunks);
        int hh = rem / n_chunks, ch = rem - hh * n_chunks;
        int r0 = ch * ATT_ROWS, nr = min(ATT_ROWS, M - r0);
        const SessDev &sd = a.sess[s];
        int P = row_pos(a, s * M);              // position of the session's first row
        int n_pos = P + r0 + nr;                // positions visible to the chunk's last row
        int lo = (int)((long long)n_pos * sp / n_splits), hi = (int)((long long)n_pos * (sp + 1) / n_splits);
        int wlo = lo + (int)((long long)(hi - lo) * wave / WAVES_PER_WG);
        int whi = lo + (int)((long long)(hi - lo) * (wave + 1) / WAVES_PER_WG);

        float q[ATT_ROWS][8], acc[ATT_ROWS][8], mx[ATT_ROWS], l[ATT_ROWS];
#pragma unroll
        for (int i = 0; i < ATT_ROWS; ++i) {
            mx[i] = ATT_NEG;
            l[i] = 0.f;
            const float *qp = a.sc.q + (size_t)(s * M + r0 + min(i, nr - 1)) * d + hh * HD + e8 * 8;
            float4 qa = *reinterpret_cast<const float4 *>(qp), qb = *reinterpret_cast<const float4 *>(qp + 4);
            q[i][0] = qa.x; q[i][1] = qa.y; q[i][2] = qa.z; q[i][3] = qa.w;
            q[i][4] = qb.x; q[i][5] = qb.y; q[i][6] = qb.z; q[i][7] = qb.w;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
        }

        for (int pb = wlo; pb < whi; pb += PPI) {
            int p = pb + grp;
            bool live = p < whi;
            int pc = live ? p : wlo;
            int page = sd.page_table[pc / KV_PAGE];
            size_t off = ((((size_t)layer * sd.n_pages + page) * H + hh) * KV_PAGE + (pc % KV_PAGE)) * HD + e8 * 8;
            uint4 kk = *reinterpret_cast<const uint4 *>(sd.kpool + off);
            uint4 vv = *reinterpret_cast<const uint4 *>(sd.vpool + off);
            float kf[8], vf[8];
            unpack8(kk, kf);
            unpack8(vv, vf);
#pragma unroll
            for (int i = 0; i < ATT_ROWS; ++i) {
                float sdot = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) sdot += q[i][e] * kf[e];
#pragma unroll
                for (int off2 = 1; off2 < LPP; off2 <<= 1) sdot += __shfl_xor(sdot, off2, 64);
                sdot *= md.att_scale;
                if (live && i < nr && p <= P + r0 + i) {
                    float nm = fmaxf(mx[i], sdot);
                    float corr = __expf(mx[i] - nm), pe = __expf(sdot - nm);
                    l[i] = l[i] * corr + pe;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][e] = acc[i][e] * corr + pe * vf[e];
                    mx[i] = nm;
                }
            }
        }
        // merge the position groups of the wave
#pragma unroll
        for (int i = 0; i < ATT_ROWS; ++i) {
#pragma unroll
            for (int off2 = LPP; off2 < 64; off2 <<= 1) {
                float om = __shfl_xor(mx[i], off2, 64), ol = __shfl_xor(l[i], off2, 64);
                float nm = fmaxf(mx[i], om);
                float c0 = __expf(mx[i] - nm), c1 = __expf(om - nm);
                l[i] = l[i] * c0 + ol * c1;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float oa = __shfl_xor(acc[i][e], off2, 64);
                    acc[i][e] = acc[i][e] * c0 + oa * c1;
                }
                mx[i] = nm;
            }
            if (grp == 0) {
                float *w = wbuf + ((size_t)wave * ATT_ROWS + i) * REC;
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e8 * 8 + e] = acc[i][e];
                if (e8 == 0) {
                    w[HD] = mx[i];
                    w[HD + 1] = l[i];
                }
            }
        }
        __syncthreads();
        // merge the waves, fixed order
        float *out = a.sc.att_part + (size_t)item * ATT_ROWS * REC;
        for (int t = tid; t < nr * REC; t += WG_THREADS) {
            int i = t / REC, e = t - i * REC;
            float gm = ATT_NEG;
            for (int w = 0; w < WAVES_PER_WG; ++w) gm = fmaxf(gm, wbuf[((size_t)w * ATT_ROWS + i) * REC + HD]);
            float r;
            if (e == HD) {
                r = gm;
            } else {
                r = 0.f;
                int src = (e == HD + 1) ? HD + 1 : e;
                for (int w = 0; w < WAVES_PER_WG; ++w) {
                    const float *wr = wbuf + ((size_t)w * ATT_ROWS + i) * REC;
                    r += wr[src] * __expf(wr[HD] - gm);
                }
            }
            out[(size_t)i * REC + e] = r;
        }
        __syncthreads();
    }
}

// merge the splits, normalise, write the attention output
__device__ void ratt_phase(const PassArgs &a)
{
    const ModelDev &md = *a.md;
    const int d = md.d, HD = md.hd, H = md.H, M = a.M, rows = a.rows;
    const int REC = HD + 2;
    const int n_chunks = (M + ATT_ROWS - 1) / ATT_ROWS, n_splits = a.att_splits;
    const int gsz = a.nwg * WG_THREADS;
    for (int it = blockIdx.x * WG_THREADS + threadIdx.x; it < rows * d; it += gsz) {
        int r = it / d, col = it - r * d;
        int s = r / M, i = r - s * M;
        int ch = i / ATT_ROWS, ii = i - ch * ATT_ROWS;
        int hh = col / HD, e = col - hh * HD;
        int unit = (s * H + hh) * n_chunks + ch;
        const float *base = a.sc.att_part + ((size_t)unit * n_splits * ATT_ROWS + ii) * REC;
        const size_t sp_stride = (size_t)ATT_ROWS * REC;
        float gm = ATT_NEG;
        for (int sp = 0; sp < n_splits; ++sp) gm = fmaxf(gm, base[sp * sp_stride + HD]);
        float num = 0.f, den = 0.f;
        for (int sp = 0; sp < n_splits; ++sp) {
            float w = __expf(base[sp * sp_stride + HD] - gm);
            num += base[sp * sp_stride + e] * w;
            den += base[sp * sp_stride + HD + 1] * w;
        }
        a.sc.attn[(size_t)r * md.Kpad_d + col] = num / den;
    }
}

// ------------------------------------------------------------------ R_GU

__device__ void rgu_phase(const PassArgs &a, char *lds)
{
    const ModelDev &md = *a.md;
    const int F = md.F, rows = a.rows;
    float *rstd = reinterpret_cast<float *>(lds);
    load_rstd(a.sc.ss_f, a.nwg, md.rows_max, rows, md.d, md.eps, rstd);
    const int gsz = a.nwg * WG_THREADS;
    for (int it = blockIdx.x * WG_THREADS + threadIdx.x; it < rows * F; it += gsz) {
        int m = it / F, f = it - m * F;
        float g = rstd[m] * reduce_out(md.gu, md.rows_max, m, f);
        float u = rstd[m] * reduce_out(md.gu, md.rows_max, m, F + f);
        float sg = g / (1.0f + __expf(-g));
        a.sc.u[(size_t)m * md.Kpad_F + f] = sg * u;
    }
}

// ------------------------------------------------------------------ heads

__device__ __forceinline__ bool cand_better(float v, int i, float bv, int bi)
{
    return v > bv || (v == bv && i < bi);
}

// logits of this workgroup's vocabulary slice, argmax candidate per row
__device__ void rhead_phase(const PassArgs &a, char *lds)
{
    const ModelDev &md = *a.md;
    const int V = md.V, rows = a.rows;
    float *rstd = reinterpret_cast<float *>(lds);
    load_rstd(a.sc.ss_a, a.nwg, md.rows_max, rows, md.d, md.eps, rstd);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int vw = (V + a.nwg - 1) / a.nwg;
    const int lo = blockIdx.x * vw, hi = min(V, lo + vw);
    float *keep = a.keep_logits ? a.sc.logits + (size_t)a.head_idx * md.rows_max * V : nullptr;
    for (int m = wave; m < rows; m += WAVES_PER_WG) {
        float bv = -INFINITY;
        int bi = 0x7FFFFFFF;
        for (int n = lo + lane; n < hi; n += 64) {
            float z = rstd[m] * reduce_out(md.head, md.rows_max, m, n);
            if (keep) keep[(size_t)m * V + n] = z;
            if (cand_better(z, n, bv, bi)) {
                bv = z;
                bi = n;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            float ov = __shfl_xor(bv, off, 64);
            int oi = __shfl_xor(bi, off, 64);
            if (cand_better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if (lane == 0) a.sc.cand[(size_t)blockIdx.x * md.rows_max + m] = make_int2(__float_as_int(bv), bi);
    }
}

// Workgroup 0: global argmax per row, accept rule per session, publication.
__device__ void accept_phase(const PassArgs &a, char *lds)
{
    if (blockIdx.x != 0) return;
    const ModelDev &md = *a.md;
    const int rows = a.rows, M = a.M;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int *tok = reinterpret_cast<int *>(lds);
    for (int m = wave; m < rows; m += WAVES_PER_WG) {
        float bv = -INFINITY;
        int bi = 0x7FFFFFFF;
        for (int g = lane; g < a.nwg; g += 64) {
            int2 c = a.sc.cand[(size_t)g * md.rows_max + m];
            float v = __int_as_float(c.x);
            if (cand_better(v, c.y, bv, bi)) {
                bv = v;
                bi = c.y;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            float ov = __shfl_xor(bv, off, 64);
            int oi = __shfl_xor(bi, off, 64);
            if (cand_better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if (lane == 0) tok[m] = bi;
    }
    __syncthreads();
    const int s = threadIdx.x;
    if (s < a.n_sess) {
        const SessDev &sd = a.sess[s];
        ee_verify_result *res = sd.result;
        const int *t = tok + s * M;
        int dev_err = __hip_atomic_load(a.sc.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (a.head_kind == HEAD_PREFILL) {
            int last = t[M - 1];
            res->next_token = last;
            res->device_status = dev_err;
            sd.state[1] = last;
        } else {
            const int gamma = M - 1;
            int delta = 0;
            while (delta < gamma && sd.drafts[delta] == t[delta]) ++delta;
            if (a.head_kind == HEAD_EXIT) {
                for (int i = 0; i < M; ++i) res->exit_tokens[a.head_idx][i] = t[i];
                res->exit_accept_len[a.head_idx] = delta;
            } else {
                for (int i = 0; i < M; ++i) res->final_tokens[i] = t[i];
                res->accept_len = delta;
                res->next_token = t[delta];
                res->device_status = dev_err;
                if (a.commit) {
                    sd.state[0] = sd.state[0] + delta + 1;
                    sd.state[1] = t[delta];
                }
            }
        }
        __threadfence_system();
    }
}

// ------------------------------------------------------------------ the segment kernel

__global__ void __launch_bounds__(WG_THREADS) ee_segment_kernel(PassArgs a)
{
    extern __shared__ __align__(16) char lds[];
    if (a.mode == 2) {  // measurement aid: layer_end grid barriers and nothing else
        for (int i = 0; i < a.layer_end; ++i) grid_barrier(a.sc.bar, a.nwg, a.sc.err, a.spin_limit);
        return;
    }
    const ModelDev &md = *a.md;
    int ph = 0;
    bool first = true;

#define EE_PHASE(body)                                                          \
    do {                                                                        \
        if (ph >= a.ph_lo && ph < a.ph_hi) {                                    \
            if (!first) grid_barrier(a.sc.bar, a.nwg, a.sc.err, a.spin_limit);  \
            first = false;                                                      \
            body;                                                               \
        }                                                                       \
        ++ph;                                                                   \
    } while (0)

    if (a.do_embed) {
        const bool head_next = (a.layer_begin == a.layer_end) && a.head_kind != HEAD_NONE;
        EE_PHASE(resid_phase<0>(a, nullptr, a.layer_begin < md.L ? md.layers[a.layer_begin].g_attn : nullptr,
                                a.layer_begin < md.L ? a.sc.xn : nullptr, head_next ? a.head_gain : nullptr,
                                head_next ? a.sc.xh : nullptr, a.sc.ss_a, lds));
    }
    for (int l = a.layer_begin; l < a.layer_end; ++l) {
        const LayerDev &lw = md.layers[l];
        EE_PHASE(gemm_dispatch(md.qkv, lw.wqkv, a.sc.xn, md.Kpad_d, a.rows, md.rows_max, a.nwg, lds));
        EE_PHASE(rqkv_phase(a, l, lds));
        if (md.hd == 128)
            EE_PHASE(att_phase<128>(a, l, lds));
        else
            EE_PHASE(att_phase<64>(a, l, lds));
        EE_PHASE(ratt_phase(a));
        EE_PHASE(gemm_dispatch(md.o, lw.wo, a.sc.attn, md.Kpad_d, a.rows, md.rows_max, a.nwg, lds));
        EE_PHASE(resid_phase<1>(a, &md.o, lw.g_ffn, a.sc.xn, nullptr, nullptr, a.sc.ss_f, lds));
        EE_PHASE(gemm_dispatch(md.gu, lw.wgu, a.sc.xn, md.Kpad_d, a.rows, md.rows_max, a.nwg, lds));
        EE_PHASE(rgu_phase(a, lds));
        EE_PHASE(gemm_dispatch(md.dn, lw.wd, a.sc.u, md.Kpad_F, a.rows, md.rows_max, a.nwg, lds));
        const bool more = l + 1 < md.L;
        const bool head_next = (l + 1 == a.layer_end) && a.head_kind != HEAD_NONE;
        EE_PHASE(resid_phase<1>(a, &md.dn, more ? md.layers[l + 1].g_attn : nullptr, more ? a.sc.xn : nullptr,
                                head_next ? a.head_gain : nullptr, head_next ? a.sc.xh : nullptr, a.sc.ss_a, lds));
    }
    if (a.head_kind != HEAD_NONE) {
        EE_PHASE(gemm_dispatch(md.head, md.wlm, a.sc.xh, md.Kpad_d, a.rows, md.rows_max, a.nwg, lds));
        EE_PHASE(rhead_phase(a, lds));
        EE_PHASE(accept_phase(a, lds));
    }
#undef EE_PHASE
}

// ------------------------------------------------------------------ load-time kernels

// row-major bf16 src[N][K] -> tiled layout (see GemmPlan); zero padding outside N x K
__global__ void tile_weights_kernel(const uint16_t *__restrict__ src, uint4 *__restrict__ dst, GemmPlan pl)
{
    const long long total = pl.T * 64;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        long long t = i >> 6;
        int lane = (int)(i & 63);
        TilePos p = tile_decode(pl, t);
        int n = p.nt * 16 + (lane & 15);
        int k0 = (p.kb * pl.KBT + p.kti) * 32 + (lane >> 4) * 8;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int k = k0 + e;
            v[e] = (n < pl.N && k < pl.K) ? src[(size_t)n * pl.K + k] : (uint16_t)0;
        }
        uint4 o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        dst[i] = o;
    }
}

__global__ void bf16_to_f32_kernel(const uint16_t *__restrict__ src, float *__restrict__ dst, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = bf16_to_f32(src[i]);
}

__global__ void set_state_kernel(int *state, int kv_len, int pending, int set_kv, int set_pending)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        if (set_kv) state[0] = kv_len;
        if (set_pending) state[1] = pending;
    }
}

// Checks the lane layout of v_mfma_f32_16x16x32_bf16 that the kernels assume:
// A[i][k] from lane (i + 16*(k/8)) element k%8, B[k][j] likewise with j, and
// D[i][j] in lane (j + 16*(i/4)) element i%4.  out[lane*4 + r] receives D.
__global__ void mfma_layout_probe_kernel(const uint4 *a, const uint4 *b, float *out)
{
    bf16x8_t A = __builtin_bit_cast(bf16x8_t, a[threadIdx.x]);
    bf16x8_t B = __builtin_bit_cast(bf16x8_t, b[threadIdx.x]);
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, B, acc, 0, 0, 0);
    for (int r = 0; r < 4; ++r) out[threadIdx.x * 4 + r] = acc[r];
}

}  // namespace ee
