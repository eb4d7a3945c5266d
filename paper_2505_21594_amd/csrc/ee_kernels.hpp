// gfx950 kernels of the verification pass.
//
// A segment of the pass (embedding, a range of layers, optionally an LM head with its
// accept step) is a list of stages.  Per layer (Eq. 3 of the paper, f = Llama-2 block)
// there are five:
//   QKV   x_hat . [Wq;Wk;Wv]^T, * rstd, RoPE, q -> scratch, k/v -> paged bf16 cache
//   ATT   causal attention of the new rows over the cache         -> attn
//   O     h += attn . Wo^T
//   GU    u = silu(rstd * x_hat.Wg^T) * (rstd * x_hat.Wu^T)
//   DN    h += u . Wd^T
// Head (z^(l) = LMHead(h^(l)); accept rule of Eq. 2 / Eq. 5; confidence of Eq. 4):
//   HEAD    x_hat . W_lm^T, * rstd, argmax candidate and softmax denominator per workgroup
//   ACCEPT  global argmax (lowest id wins ties), confidence, accept length, publication
//           to pinned host memory, KV commit.
// By default every stage is one launch (ee_gemm_chain_kernel for the five GEMM kinds,
// ee_att_kernel, ee_misc_kernel for embedding and accept); optionally consecutive GEMM
// stages share one launch of ee_gemm_chain_kernel with a grid-wide barrier between them,
// each wave fetching the first weight tiles of its next stage before it enters the barrier.
//
// Every GEMM stage streams the weights once (HBM-bound).  A workgroup owns whole
// n-tiles for the full K, so its outputs are complete after a cross-wave sum in
// LDS and the element-wise epilogue runs in the same stage.  RMSNorm is split:
// the GEMM input is g * h (written by the stage that produces h), the row factor
// rstd = 1/sqrt(mean(h^2)+eps), from per-workgroup partial sums, multiplies the fp32 result.
#pragma once

#include "ee_device.hpp"

namespace ee {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

constexpr int D = PF_DEPTH;

// Pointers read from descriptors in memory are generic to the compiler, and generic loads go
// through the flat path, whose completion also counts against the LDS counter: a wait for an
// LDS read would then drain every weight load in flight.  These helpers state that the
// address is global memory.
#define EE_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ const EE_GLOBAL T *as_global(const T *p)
{
    return (const EE_GLOBAL T *)(p);
}
// The same for stores.  One generic (flat) access anywhere in a kernel also makes the compiler
// treat the order of returning loads as unknown and wait for all of them at every use.
template <typename T>
__device__ __forceinline__ EE_GLOBAL T *as_global_mut(T *p)
{
    return (EE_GLOBAL T *)(p);
}

// 16-byte weight load of a tile: buffer load with the stage's weights as the resource, the
// lane's 16 bytes as the vector offset and the tile's byte offset as the scalar offset, so the
// stream needs no per-tile address arithmetic in vector registers.  Plain cache policy: on
// this part non-temporal loads measured about 10 % slower for the same access pattern.
typedef __amdgpu_buffer_rsrc_t WRes;
__device__ __forceinline__ WRes weight_resource(const uint4 *W)
{
    // raw buffer, no stride, maximal range (offsets stay inside the stage's allocation).  The
    // pointer is the same in every lane; saying so keeps the resource in scalar registers.
    const unsigned long long p = reinterpret_cast<unsigned long long>(W);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)p), hi = __builtin_amdgcn_readfirstlane((unsigned)(p >> 32));
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(((unsigned long long)hi << 32) | lo), 0, 0x7FFFFFFF, 0x00020000);
}
__device__ __forceinline__ uint4 load_tile16(WRes r, int lane_off, int tile_off)
{
    u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, tile_off, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ uint4 load_global16(const void *p)
{
    u32x4_t v = *as_global(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// Device-scope accesses for the small buffers that cross a grid barrier inside one launch
// (GEMM inputs written by one stage's epilogue and read by the next stage's staging, partial
// sums of squares).  Stores write through to memory and loads bypass the per-XCD L2, so the
// barrier itself needs no cache write-back or invalidate; everything else is read-only in
// the launch or crosses a kernel boundary.
__device__ __forceinline__ void store_dev64(void *p, uint2 v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), ((unsigned long long)v.y << 32) | v.x,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_dev32(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_dev32(const float *p)
{
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The value itself, but opaque to the optimiser: keeps per-thread index arithmetic of a stage
// from being hoisted out of the stage loop, where it would occupy registers for the whole kernel.
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}
// debug: stamp slot (stage-in-launch, k) with the 100 MHz wall clock, workgroup 0 only
#define EE_TRACE_SLOTS 8
#define EE_TRACE_WG_BASE (1 << 14)  // per-workgroup stamps follow workgroup 0's slots
__device__ __forceinline__ void trace_stamp(const PassArgs &a, int stage_in_launch, int k)
{
    if (a.sc.trace && blockIdx.x == 0 && threadIdx.x == 0)
        a.sc.trace[a.trace_base + stage_in_launch * EE_TRACE_SLOTS + k] = wall_clock64();
}
// debug: every workgroup stamps the start (k = 0) and the end (k = 1) of the launch
__device__ __forceinline__ void trace_stamp_wg(const PassArgs &a, int k)
{
    if (a.sc.trace && threadIdx.x == 0)
        a.sc.trace[EE_TRACE_WG_BASE + ((size_t)(a.trace_base / EE_TRACE_SLOTS) * a.nwg + blockIdx.x) * 2 + k] = wall_clock64();
}
// The launch arguments are several hundred bytes; the compiler fetches their fields where it
// needs them, and every first touch of another 64-byte line is a miss of the scalar cache that
// the wave has to wait out: about 0.22 us each, eight or more in a row at the start of every
// launch.  This reads one word of every line at once, so the misses overlap, and returns the
// argument block through a pointer the compiler cannot trace back, so that none of its own
// fetches can be scheduled before these.
template <int LINE, int LINES>
__device__ __forceinline__ void warm_line(unsigned long long ka)
{
    if constexpr (LINE < LINES) {
        unsigned t;
        asm volatile("s_load_dword %0, %1, %2" : "=s"(t) : "s"(ka), "n"(LINE * 64) : "memory");
        warm_line<LINE + 1, LINES>(ka);
    }
}
__device__ __forceinline__ const PassArgs &warmed_arguments()
{
    unsigned long long ka = reinterpret_cast<unsigned long long>((const void *)__builtin_amdgcn_kernarg_segment_ptr());
    warm_line<0, (sizeof(PassArgs) + 63 - 4) / 64>(ka);  // last word read lies inside the block
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(ka)::"memory");
    return *(const PassArgs *)(const __attribute__((address_space(4))) PassArgs *)ka;
}
// all vector memory operations of this wave have completed
// (the builtin, not inline assembly: the compiler's own bookkeeping of loads in flight sees it,
// so code after it is not made to wait again for loads that this wait has already covered)
__device__ __forceinline__ void wait_vmem()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even; inputs are finite
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// ------------------------------------------------------------------ grid barrier

// Every workgroup publishes the epoch it has reached in its own flag and waits until all
// flags have reached it.  Callers make their cross-workgroup data visible themselves:
// device-scope stores followed by wait_vmem() in every wave before the barrier, device-scope
// loads after it.  The wait is bounded: after spin_limit polls the workgroup raises *err and
// goes on, and later barriers fall through at once, so the grid always drains.
__device__ __forceinline__ void grid_barrier(unsigned *flags, unsigned nwg, unsigned epoch, int *err,
                                             unsigned spin_limit)
{
    wait_vmem();
    __syncthreads();
    if (threadIdx.x < 64) {
        if (threadIdx.x == 0)
            __hip_atomic_store(&flags[blockIdx.x], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        while (true) {
            bool ok = true;
            for (unsigned i = threadIdx.x; i < nwg; i += 64) {
                unsigned f = __hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = ok && ((int)(f - epoch) >= 0);
            }
            if (__all(ok)) break;
            ++spins;
            if ((spins & 63u) == 0 &&
                __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                break;
            if (spins > spin_limit) {
                __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
    }
    __syncthreads();
}

// ------------------------------------------------------------------ rows

// Fields of session s's descriptor.  Session 0's descriptor also travels by value in the launch
// arguments, so the common one-session pass needs no load from memory to find them.
// (written so that the two sources are never merged into one pointer of unknown address space)
template <typename T>
__device__ __forceinline__ T sess_pick(bool first, const T &own, const T *other)
{
    T v = own;
    if (!first) v = *as_global(other);
    return v;
}
#define EE_SESS(a, s, field) sess_pick((s) == 0, (a).sess0.field, &(a).sess[s].field)

__device__ __forceinline__ int row_pos(const PassArgs &a, int r)
{
    if (a.mode == 1) return a.pf_pos0 + r;
    int s = r / a.M;
    return EE_SESS(a, s, kv_len) + (r - s * a.M);
}

__device__ __forceinline__ int row_token(const PassArgs &a, int r)
{
    if (a.mode == 1) return a.pf_tokens[r];
    int s = r / a.M, i = r - s * a.M;
    return i == 0 ? EE_SESS(a, s, pending) : EE_SESS(a, s, drafts)[i - 1];
}

// ------------------------------------------------------------------ LDS map

struct Misc {  // views into the misc region of the LDS block
    float *rstd;       // [rows_max]
    float *rowss;      // [rows_max]  this workgroup's sum of h^2 per row (O / DN stages)
    int *pos;          // [rows_max]
    long long *kvoff;  // [rows_max]  element offset of the row's (layer, page, head 0) record in the KV pools
    float2 *rope;      // [rows_max][hd/2]
    float *bestv;      // [rows_max]
    int *besti;        // [rows_max]
    float *sume;       // [rows_max]  sum of exp(logit - bestv) over the columns seen so far
};

__device__ __forceinline__ Misc misc_views(const ModelDev &md, const GemmPlan &pl, char *lds)
{
    Misc m;
    char *p = lds + pl.lds_misc_off;
    const int R = md.rows_max;
    m.kvoff = reinterpret_cast<long long *>(p);
    p += (size_t)R * 8;
    m.rope = reinterpret_cast<float2 *>(p);
    p += (size_t)R * (md.hd / 2) * 8;
    m.rstd = reinterpret_cast<float *>(p);
    p += (size_t)R * 4;
    m.rowss = reinterpret_cast<float *>(p);
    p += (size_t)R * 4;
    m.pos = reinterpret_cast<int *>(p);
    p += (size_t)R * 4;
    m.bestv = reinterpret_cast<float *>(p);
    p += (size_t)R * 4;
    m.besti = reinterpret_cast<int *>(p);
    p += (size_t)R * 4;
    m.sume = reinterpret_cast<float *>(p);
    return m;
}

// ------------------------------------------------------------------ weight-stream geometry

struct Seg {  // one (group, K-block) of a workgroup's tile sequence, seen from one wave
    int gn;           // n-tiles in the group
    int klen, kst;    // k-tiles of the block, first k-tile
    int s0, slen;     // this wave's slice of every run: [s0, s0 + slen)
    int n;            // tiles of this wave in the segment = gn * slen
    int step0;        // position of the segment's first tile in this wave's sequence
};

__device__ __forceinline__ void wg_units(const GemmPlan &pl, int nwg, int g, int &nt0, int &n_local)
{
    int u0 = 0, u1 = 0;
    if (g < nwg) unit_range(pl.U, nwg, g, u0, u1);  // workgroups past the stage's count own nothing
    nt0 = u0 * pl.tpu;
    n_local = (u1 - u0) * pl.tpu;
}

// tiles this wave streams in the groups/blocks before (gi, kb)
__device__ __forceinline__ int seg_steps_before(const GemmPlan &pl, int n_local, int wave, int gi, int kb)
{
    // every full pass over K gives the wave  sum_kb slen(kb)  tiles per n-tile
    int per_tile = 0, before_kb = 0;
    for (int b = 0; b < pl.nKB; ++b) {
        int kst = pl.KT * b / pl.nKB, klen = pl.KT * (b + 1) / pl.nKB - kst;
        int sl = klen * (wave + 1) / WAVES - klen * wave / WAVES;
        per_tile += sl;
        if (b < kb) before_kb += sl;
    }
    const int gn = min(pl.GRP, n_local - gi * pl.GRP);
    return gi * pl.GRP * per_tile + gn * before_kb;
}

__device__ __forceinline__ Seg seg_setup(const GemmPlan &pl, int nt0, int n_local, int wave, int gi, int kb)
{
    Seg s;
    s.gn = min(pl.GRP, n_local - gi * pl.GRP);
    s.kst = pl.KT * kb / pl.nKB;
    s.klen = pl.KT * (kb + 1) / pl.nKB - s.kst;
    s.s0 = s.klen * wave / WAVES;
    s.slen = s.klen * (wave + 1) / WAVES - s.s0;
    s.n = s.gn * s.slen;
    s.step0 = seg_steps_before(pl, n_local, wave, gi, kb);
    return s;
}

// byte offset of the wave's tile number `step` (see GemmPlan): slot (step*nwg + g)*WAVES + wave;
// at most the stage's bytes, below 2^31
__device__ __forceinline__ int tile_off(int nwg, int wave, int step)
{
    return ((step * nwg + (int)blockIdx.x) * WAVES + wave) * 1024;
}

// first min(D, s.n) tiles of the wave's sequence in segment s
__device__ __forceinline__ void seg_prefetch(const uint4 *__restrict__ W, int nwg, int wave, const Seg &s, uint4 (&pre)[D])
{
    const WRes res = weight_resource(W);
    const int lane_off = (threadIdx.x & 63) * 16;
#pragma unroll
    for (int j = 0; j < D; ++j)
        if (j < s.n) pre[j] = load_tile16(res, lane_off, tile_off(nwg, wave, s.step0 + j));
}

struct NextGemm {  // the GEMM stage that follows in the same launch
    const GemmPlan *pl;  // in device memory; nullptr: nothing to fetch
    const uint4 *W;
};

__device__ __forceinline__ bool prefetch_stage(const NextGemm &nx, int nwg, uint4 (&pre)[D])
{
    if (!nx.pl) return false;
    int nt0, n_local;
    wg_units(*nx.pl, nx.pl->nwg, blockIdx.x, nt0, n_local);
    if (n_local == 0) return true;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    Seg s = seg_setup(*nx.pl, nt0, n_local, wave, 0, 0);
    seg_prefetch(nx.W, nx.pl->nwg, wave, s, pre);
    return true;
}

// ------------------------------------------------------------------ GEMM stage


struct GemmIn {
    const uint16_t *x;  // the input (already scaled by the norm gain) as two bf16 terms, k-tile-major (x_index)
    const float *ss;    // [nwg][rows_max] partial sums of squares for rstd, or nullptr
};

// GEMM inputs are stored the way the stages consume them: [k-tile][term][row][32] bf16 with
// `rows` = the rows of this pass, term 0 = hi, 1 = lo.  The k-slice one wave multiplies with
// (all rows, both terms) is then one contiguous range, which a few 1 KB loads copy into LDS,
// and the 16 rows x 4 quads of one MFMA operand read one contiguous kilobyte of LDS.
__device__ __forceinline__ size_t x_index(int rows, int m, int k, int term)
{
    return ((size_t)((k >> 5) * 2 + term) * rows + m) * 32 + (k & 31);
}

// split x into two bf16 terms: hi = bf16(x), lo = bf16(x - hi).  The MFMA takes bf16 operands;
// feeding both terms keeps about 16 mantissa bits of the activations (weights are exact
// bf16).  The matrix cores idle most of the time in the HBM-bound loop, so the second MFMA
// per tile is free.
__device__ __forceinline__ void split_bf16(float x, uint32_t &hi, uint32_t &lo)
{
    hi = f32_to_bf16(x);
    lo = f32_to_bf16(x - __uint_as_float(hi << 16));
}

// four consecutive columns k .. k+3 (k a multiple of 4) of row m
__device__ __forceinline__ void store_split4(uint16_t *x, int rows, int m, int k, const float *v)
{
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_bf16(v[e], h[e], l[e]);
    store_dev64(x + x_index(rows, m, k, 0), make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16)));
    store_dev64(x + x_index(rows, m, k, 1), make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16)));
}

// Wave-private staging of the GEMM input: the wave copies the k-slice it multiplies with,
// k-tiles [kst + s0, kst + s0 + slen) of every row and of both bf16 terms: one contiguous range
// in memory, copied straight into LDS at the same offset relative to the K-block's start.  No
// registers hold the data and no other wave reads this slice, so no workgroup barrier is
// needed: the wave waits for its own loads (wait_vmem) and goes on.  One load instruction
// moves 64 x 16 bytes.  DEV = true reads with device scope (the input was written earlier in
// the same launch by other workgroups).
#define EE_LDS __attribute__((address_space(3)))
template <bool DEV>
__device__ __forceinline__ void stage_x_wave(const GemmIn &in, int rows, int kst, int s0, int slen, char *lds, int lane)
{
    const size_t tile_elems = (size_t)2 * rows * 32;          // one k-tile: both terms, all rows
    const uint16_t *src = in.x + (size_t)(kst + s0) * tile_elems;
    char *dst = lds + (size_t)s0 * tile_elems * 2;
    const int nchunk = slen * 2 * rows * 4;                     // 16-byte chunks of the slice
    for (int c0 = 0; c0 < nchunk; c0 += 64)
        if (c0 + lane < nchunk)
            __builtin_amdgcn_global_load_lds((const EE_GLOBAL void *)(src + (size_t)(c0 + lane) * 8),
                                             (EE_LDS void *)(dst + (size_t)c0 * 16), 16, 0, DEV ? 16 : 0);
}

// rstd[m] = 1/sqrt(sum_g ss[g][m] / d + eps) into LDS, fixed summation order.  DEV: the partial
// sums were written earlier in the same launch (device-scope loads); otherwise ordinary loads,
// which the XCD's L2 serves to all but the first workgroup: every workgroup reads the same
// few kilobytes, and past the L2 that is thousands of requests for the same lines.
template <bool DEV>
__device__ __forceinline__ void load_rstd(const float *ss, int nwg, int rows_max, int rows, int d, float eps,
                                          float *rstd_lds)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int m = wave; m < rows; m += WAVES) {
        float s = 0.f;
        for (int g = lane; g < nwg; g += 64)
            s += DEV ? load_dev32(ss + (size_t)g * rows_max + m) : *as_global(ss + (size_t)g * rows_max + m);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) rstd_lds[m] = 1.0f / sqrtf(s / (float)d + eps);
    }
}

__device__ __forceinline__ bool cand_better(float v, int i, float bv, int bi)
{
    return v > bv || (v == bv && i < bi);
}

// Epilogue of one group: sum the waves' partial tiles, apply the stage's element-wise tail.
struct GemmEpi {           // what the O / DN epilogue produces besides h
    const float *gain_xn;  // gain of the next GEMM input (xn), or nullptr
    const float *gain_xh;  // gain of the LM-head input (xh), or nullptr
    float *ss_out;         // [nwg][rows_max] partial sums of h^2
};

__device__ __forceinline__ void gemm_epilogue(const PassArgs &a, int kind, int layer, const GemmPlan &pl, int nt_first,
                                              int gn, int rows, const GemmEpi &ep, const Misc &mi, char *lds)
{
    const ModelDev &md = a.mdv;
    const float *slots = reinterpret_cast<const float *>(lds + pl.lds_slots_off);
    const int tid = opaque(threadIdx.x);
    const size_t wstride = (size_t)pl.GRP * rows * 16;  // floats per wave in the slot buffer
    const int n_part = pl.shared_acc ? 1 : WAVES;        // partial tiles to sum per output tile
    if (kind == G_GU) {
        const int items = (gn >> 1) * rows * 4;
        for (int idx = tid; idx < items; idx += WG_THREADS) {
            int p = idx / (rows * 4), rem = idx - p * rows * 4;
            int m = rem >> 2, qd = rem & 3;
            const float *sg = slots + ((size_t)(2 * p) * rows + m) * 16 + qd * 4;
            const float *su = sg + (size_t)rows * 16;
            float4 G = make_float4(0.f, 0.f, 0.f, 0.f), U = G;
#pragma unroll 2
            for (int w = 0; w < n_part; ++w) {
                float4 x = *reinterpret_cast<const float4 *>(sg + w * wstride);
                float4 y = *reinterpret_cast<const float4 *>(su + w * wstride);
                G.x += x.x; G.y += x.y; G.z += x.z; G.w += x.w;
                U.x += y.x; U.y += y.y; U.z += y.z; U.w += y.w;
            }
            const float rs = mi.rstd[m];
            float g[4] = {G.x * rs, G.y * rs, G.z * rs, G.w * rs}, u[4] = {U.x * rs, U.y * rs, U.z * rs, U.w * rs};
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = g[e] / (1.0f + __expf(-g[e])) * u[e];
            const int f = ((nt_first >> 1) + p) * 16 + qd * 4;
            store_split4(a.sc.u, rows, m, f, o);
        }
        return;
    }
    float *zbuf = reinterpret_cast<float *>(lds + pl.lds_zbuf_off);  // head: [rows][GRP*16] logits of this group; O/DN: squares
    const int items = gn * rows * 4;
    for (int idx = tid; idx < items; idx += WG_THREADS) {
        int ntg = idx / (rows * 4), rem = idx - ntg * rows * 4;
        int m = rem >> 2, qd = rem & 3;
        const float *sp = slots + ((size_t)ntg * rows + m) * 16 + qd * 4;
        float4 S = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
        for (int w = 0; w < n_part; ++w) {
            float4 x = *reinterpret_cast<const float4 *>(sp + w * wstride);
            S.x += x.x; S.y += x.y; S.z += x.z; S.w += x.w;
        }
        const int n = (nt_first + ntg) * 16 + qd * 4;  // four consecutive output columns
        if (kind == G_O || kind == G_DN) {
            float sq = 0.f;
            if (n < md.d) {
                float4 *hp = reinterpret_cast<float4 *>(a.sc.h + (size_t)m * md.d + n);
                float4 hv = *hp;
                float v[4] = {hv.x + S.x, hv.y + S.y, hv.z + S.z, hv.w + S.w};
                *hp = make_float4(v[0], v[1], v[2], v[3]);
                sq = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                if (ep.gain_xn) {
                    float4 g = *reinterpret_cast<const float4 *>(ep.gain_xn + n);
                    float x[4] = {v[0] * g.x, v[1] * g.y, v[2] * g.z, v[3] * g.w};
                    store_split4(a.sc.xn, rows, m, n, x);
                }
                if (ep.gain_xh) {
                    float4 g = *reinterpret_cast<const float4 *>(ep.gain_xh + n);
                    float x[4] = {v[0] * g.x, v[1] * g.y, v[2] * g.z, v[3] * g.w};
                    store_split4(a.sc.xh, rows, m, n, x);
                }
            }
            zbuf[idx] = sq;  // (ntg, m, quad) order
        } else if (kind == G_QKV) {
            const int d = md.d, hd = md.hd;
            const float rs = mi.rstd[m];
            float v[4] = {S.x * rs, S.y * rs, S.z * rs, S.w * rs};
            const int sect = n / d, c = n - sect * d;
            const int head = c / hd, e = c - head * hd;
            if (sect < 2) {
                // columns are pair-interleaved inside a head: (e, e+1) = RoPE pair e/2
                float2 c0 = mi.rope[m * (hd >> 1) + (e >> 1)], c1 = mi.rope[m * (hd >> 1) + (e >> 1) + 1];
                float y0 = v[0] * c0.x - v[1] * c0.y, y1 = v[1] * c0.x + v[0] * c0.y;
                float y2 = v[2] * c1.x - v[3] * c1.y, y3 = v[3] * c1.x + v[2] * c1.y;
                v[0] = y0; v[1] = y1; v[2] = y2; v[3] = y3;
            }
            if (sect == 0) {
                *reinterpret_cast<float4 *>(a.sc.q + (size_t)m * d + c) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
                // cached value = hi + lo, two bf16 terms.  K: [position][term][hd]; V transposed
                // inside the page: [term][hd][position] (see the attention stage)
                const int ses = a.mode == 1 ? 0 : m / a.M;
                uint32_t vh[4], vl[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) split_bf16(v[t], vh[t], vl[t]);
                const size_t rec = mi.kvoff[m] + (size_t)head * KV_PAGE * 2 * hd;  // this (page, head) record
                const int slot = mi.pos[m] % KV_PAGE;
                if (sect == 1) {
                    EE_GLOBAL uint16_t *kr = as_global_mut(EE_SESS(a, ses, kpool)) + rec + (size_t)slot * 2 * hd + e;
                    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
                    *reinterpret_cast<EE_GLOBAL u32x2_t *>(kr) = (u32x2_t){vh[0] | (vh[1] << 16), vh[2] | (vh[3] << 16)};
                    *reinterpret_cast<EE_GLOBAL u32x2_t *>(kr + hd) = (u32x2_t){vl[0] | (vl[1] << 16), vl[2] | (vl[3] << 16)};
                } else {
                    EE_GLOBAL uint16_t *vr = as_global_mut(EE_SESS(a, ses, vpool)) + rec + slot;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        vr[(size_t)(e + t) * KV_PAGE] = (uint16_t)vh[t];
                        vr[(size_t)(hd + e + t) * KV_PAGE] = (uint16_t)vl[t];
                    }
                }
            }
        } else {  // G_HEAD
            const float rs = mi.rstd[m];
            float z[4] = {S.x * rs, S.y * rs, S.z * rs, S.w * rs};
            float *zr = zbuf + (size_t)m * pl.GRP * 16 + ntg * 16 + qd * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (n + e >= md.V) z[e] = -INFINITY;
                zr[e] = z[e];
            }
            if (a.keep_logits) {
                float *keep = a.sc.logits + ((size_t)a.head_idx * md.rows_max + m) * md.V;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n + e < md.V) keep[n + e] = z[e];
            }
        }
    }
    if (kind == G_O || kind == G_DN) {
        __syncthreads();
        if (tid < rows) {  // this group's sum of squares per row, fixed order
            float t = 0.f;
            for (int ntg = 0; ntg < gn; ++ntg)
                for (int qd = 0; qd < 4; ++qd) t += zbuf[(ntg * rows + tid) * 4 + qd];
            mi.rowss[tid] += t;
        }
    }
    if (kind == G_HEAD) {
        __syncthreads();
        const int lane = tid & 63, wave = tid >> 6;
        for (int m = wave; m < rows; m += WAVES) {
            float bv = -INFINITY;
            int bi = 0x7FFFFFFF;
            for (int c = lane; c < gn * 16; c += 64) {
                float z = zbuf[(size_t)m * pl.GRP * 16 + c];
                int n = nt_first * 16 + c;
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
            // sum of exp(z - bv) over the group's columns (masked columns hold -inf and add 0):
            // the softmax denominator for the confidence score (paper Eq. 4), kept relative to the
            // running maximum like the argmax candidate
            float se = 0.f;
            for (int c = lane; c < gn * 16; c += 64) se += __expf(zbuf[(size_t)m * pl.GRP * 16 + c] - bv);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) se += __shfl_xor(se, off, 64);
            if (lane == 0 && bv > -INFINITY) {  // (a group of masked columns only contributes nothing)
                const float ov = mi.bestv[m];
                if (cand_better(bv, bi, ov, mi.besti[m])) {
                    mi.sume[m] = mi.sume[m] * __expf(ov - bv) + se;  // exp(-inf) = 0 the first time
                    mi.bestv[m] = bv;
                    mi.besti[m] = bi;
                } else {
                    mi.sume[m] += se * __expf(bv - ov);
                }
            }
        }
    }
}

template <int MT>
__device__ void gemm_stage_t(const PassArgs &a, int kind, int layer, const GemmPlan pl, const uint4 *__restrict__ W,
                             const GemmIn &in, const GemmEpi &ep, uint4 (&buf)[D], bool &have_pre, const NextGemm &next,
                             char *lds, int tsi)
{
    const ModelDev &md = a.mdv;
    const int tid = opaque(threadIdx.x), lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rows = a.rows;
    const Misc mi = misc_views(md, pl, lds);
    int nt0, n_local;
    wg_units(pl, pl.nwg, blockIdx.x, nt0, n_local);

    if (kind == G_HEAD) {
        if (tid < rows) {
            mi.bestv[tid] = -INFINITY;
            mi.besti[tid] = 0x7FFFFFFF;
            mi.sume[tid] = 0.f;
        }
    }
    if (n_local == 0) {  // nothing to stream here (uniform over the workgroup)
        have_pre = prefetch_stage(next, a.nwg, buf);
        if (kind == G_HEAD && tid < rows) {
            store_dev64(a.sc.cand + (size_t)blockIdx.x * md.rows_max + tid, make_uint2(__float_as_uint(-INFINITY), 0x7FFFFFFFu));
            store_dev32(a.sc.cand_sum + (size_t)blockIdx.x * md.rows_max + tid, 0.f);
        }
        if ((kind == G_O || kind == G_DN) && tid < rows) store_dev32(ep.ss_out + (size_t)blockIdx.x * md.rows_max + tid, 0.f);
        return;
    }
    if ((kind == G_O || kind == G_DN) && tid < rows) mi.rowss[tid] = 0.f;
    if (pl.shared_acc) {  // the accumulators start at zero (one workgroup barrier before the first add)
        float *acc0 = reinterpret_cast<float *>(lds + pl.lds_slots_off);
        for (int i = tid; i < n_local * rows * 16; i += WG_THREADS) acc0[i] = 0.f;
        __syncthreads();
    }
    trace_stamp(a, tsi, 0);
    // start the weight stream before anything else (unless the previous stage already did)
    if (!have_pre) seg_prefetch(W, pl.nwg, wave, seg_setup(pl, nt0, n_local, wave, 0, 0), buf);
    const uint16_t *xs = reinterpret_cast<const uint16_t *>(lds);  // the K-block's input, [k-tile][term][row][32]
    float *slots = reinterpret_cast<float *>(lds + pl.lds_slots_off);
    int brow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) brow[mt] = min(mt * 16 + (lane & 15), rows - 1) * 32;
    const int bk = (lane >> 4) * 8;
    const int n_groups = (n_local + pl.GRP - 1) / pl.GRP;

    for (int gi = 0; gi < n_groups; ++gi) {
        const int gn = min(pl.GRP, n_local - gi * pl.GRP);
        for (int kb = 0; kb < pl.nKB; ++kb) {
            const Seg s = seg_setup(pl, nt0, n_local, wave, gi, kb);
            const bool restage = pl.nKB > 1 || gi == 0;
            if (restage) {
                // A wave overwrites only its own slice of the previous block when every block has
                // the same length (the slices then coincide); otherwise slices shift between
                // blocks and the other waves must be done with theirs first.
                if ((gi > 0 || kb > 0) && pl.KT % pl.nKB != 0) __syncthreads();
                if (a.ph_hi - a.ph_lo > 1)
                    stage_x_wave<true>(in, rows, s.kst, s.s0, s.slen, lds, lane);
                else  // the input comes from an earlier launch: ordinary loads, served by the XCD's L2
                    stage_x_wave<false>(in, rows, s.kst, s.s0, s.slen, lds, lane);
                if (in.ss && gi == 0 && kb == 0) {
                    if (a.ph_hi - a.ph_lo > 1)
                        load_rstd<true>(in.ss, a.nwg, md.rows_max, rows, pl.K, md.eps, mi.rstd);
                    else
                        load_rstd<false>(in.ss, a.nwg, md.rows_max, rows, pl.K, md.eps, mi.rstd);
                }
                if (kind == G_QKV && gi == 0 && kb == 0) {
                    // per-row position, KV record and RoPE factors for the epilogue (read after the
                    // workgroup barrier that precedes it)
                    if (tid < rows) {
                        const int m = tid;
                        const int pos = row_pos(a, m);
                        const int ses = a.mode == 1 ? 0 : m / a.M;
                        const int cbase = EE_SESS(a, ses, contig_base);
                        const int page = cbase >= 0 ? cbase + pos / KV_PAGE : as_global(EE_SESS(a, ses, page_table))[pos / KV_PAGE];
                        mi.pos[m] = pos;
                        mi.kvoff[m] = (((long long)layer * EE_SESS(a, ses, n_pages) + page) * md.H) * KV_PAGE * 2 * md.hd;  // record of head 0
                    }
                    const int half = md.hd >> 1;
                    for (int i = tid; i < rows * half; i += WG_THREADS) {
                        int m = i / half, j = i - m * half;
                        const int ses = a.mode == 1 ? 0 : m / a.M;
                        const unsigned long long cs = *as_global(reinterpret_cast<const unsigned long long *>(EE_SESS(a, ses, rope) + (size_t)row_pos(a, m) * half + j));
                        mi.rope[i] = make_float2(__uint_as_float((unsigned)cs), __uint_as_float((unsigned)(cs >> 32)));
                    }
                }
                wait_vmem();  // this wave's slice is in LDS (and its first weight tiles have arrived)
                trace_stamp(a, tsi, 1 + min(kb, 1));
            }

            // ---- this wave's tiles of the segment
            f32x4_t acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
            if (s.slen == 0 && kb == 0 && !pl.shared_acc) {  // no tiles in this block: contribute zeros
                for (int ntg = 0; ntg < gn; ++ntg)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        int m = mt * 16 + (lane & 15);
                        if (m < rows)
                            *reinterpret_cast<float4 *>(slots + (((size_t)wave * pl.GRP + ntg) * rows + m) * 16 + (lane >> 4) * 4) =
                                make_float4(0.f, 0.f, 0.f, 0.f);
                    }
            }
            int ntg = 0, kk = 0;  // compute cursor
            const WRes wres = weight_resource(W);
            const int lane_off = lane * 16;
            const int woff = tile_off(pl.nwg, wave, s.step0);
            const int wstep = pl.nwg * WAVES * 1024;  // bytes from one tile of the wave's sequence to the next
            const int woff_last = woff + (s.n - 1) * wstep;
            // one tile: two MFMAs (both bf16 terms of the input); at the end of an n-tile's run
            // the partial tile goes to the wave's slot in LDS
            auto tile_step = [&](const uint4 &av) __attribute__((always_inline)) {
                bf16x8_t A = __builtin_bit_cast(bf16x8_t, av);
                const int xo = (s.s0 + kk) * 2 * rows * 32 + bk;  // this k-tile's hi rows; the lo rows follow them
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    uint4 bh = *reinterpret_cast<const uint4 *>(xs + brow[mt] + xo);
                    uint4 bl = *reinterpret_cast<const uint4 *>(xs + brow[mt] + xo + rows * 32);
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8_t, bh), acc[mt], 0, 0, 0);
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8_t, bl), acc[mt], 0, 0, 0);
                }
                if (++kk == s.slen) {
                    // D layout: lane holds rows (lane>>4)*4 .. +3 of N, column (lane&15) of M
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        int m = mt * 16 + (lane & 15);
                        if (m < rows) {
                            if (pl.shared_acc) {
                                EE_LDS float *dst = (EE_LDS float *)(slots + ((size_t)ntg * rows + m) * 16 + (lane >> 4) * 4);
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    __hip_atomic_fetch_add(dst + r, acc[mt][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            } else {
                                float4 *dst = reinterpret_cast<float4 *>(
                                    slots + (((size_t)wave * pl.GRP + ntg) * rows + m) * 16 + (lane >> 4) * 4);
                                float4 v = make_float4(acc[mt][0], acc[mt][1], acc[mt][2], acc[mt][3]);
                                if (kb > 0) {
                                    float4 o = *dst;
                                    v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                                }
                                *dst = v;
                            }
                        }
                        acc[mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                    }
                    kk = 0;
                    ++ntg;
                }
            };
            // Full blocks of D tiles: every load is unconditional (the look-ahead is clamped to
            // the segment's last tile), so the compiler can count the loads in flight and each
            // use waits for exactly its own tile.  Loads under a condition make it wait for all
            // of them, which halves what one wave can pull.
            // Nothing may be in flight when the loop is entered, else (e.g. with the stores
            // of an earlier epilogue still counted) the compiler falls back to waiting for all.
            wait_vmem();
            int i = 0;
            for (; i + D <= s.n; i += D) {
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    // use the tile, then refill its registers: issuing the load first would need a
                    // second set of registers and a copy (with a wait) at the end of the block
                    tile_step(buf[j]);
                    buf[j] = load_tile16(wres, lane_off, min(woff + (i + j + D) * wstep, woff_last));
                }
            }
#pragma unroll
            for (int j = 0; j < D; ++j)
                if (i + j < s.n) tile_step(buf[j]);
            // ---- fetch ahead: next segment of this stage, or the first tiles of the next GEMM stage
            const bool last_seg = (gi == n_groups - 1) && (kb == pl.nKB - 1);
            if (!last_seg) {
                const int ngi = kb + 1 < pl.nKB ? gi : gi + 1, nkb = kb + 1 < pl.nKB ? kb + 1 : 0;
                const Seg ns = seg_setup(pl, nt0, n_local, wave, ngi, nkb);
                seg_prefetch(W, pl.nwg, wave, ns, buf);
            } else {
                have_pre = prefetch_stage(next, a.nwg, buf);
            }
        }
        trace_stamp(a, tsi, 3);
        __syncthreads();
        trace_stamp(a, tsi, 4);
        gemm_epilogue(a, kind, layer, pl, nt0 + gi * pl.GRP, gn, rows, ep, mi, lds);
        trace_stamp(a, tsi, 5);
        if (gi + 1 < n_groups) __syncthreads();
    }
    if (kind == G_O || kind == G_DN) {
        __syncthreads();
        if (tid < rows) store_dev32(ep.ss_out + (size_t)blockIdx.x * md.rows_max + tid, mi.rowss[tid]);
    }
    if (kind == G_HEAD) {
        __syncthreads();
        if (tid < rows) {  // device-scope stores: the accept step may run in another workgroup of this launch
            store_dev64(a.sc.cand + (size_t)blockIdx.x * md.rows_max + tid, make_uint2(__float_as_uint(mi.bestv[tid]), (unsigned)mi.besti[tid]));
            store_dev32(a.sc.cand_sum + (size_t)blockIdx.x * md.rows_max + tid, mi.sume[tid]);
        }
    }
}

// ------------------------------------------------------------------ embedding

// h = embedding of each row's token (or the supplied embedding row); workgroup g owns the
// columns [g*cw, (g+1)*cw) and also emits the first layer's GEMM input and its share of h^2
__device__ void embed_stage(const PassArgs &a, char *lds)
{
    const ModelDev &md = a.mdv;
    const int d = md.d, rows = a.rows, tid = threadIdx.x;
    const int cw = ((d + a.nwg - 1) / a.nwg + 3) & ~3;  // columns per workgroup, multiple of 4
    const int n0 = blockIdx.x * cw;
    const int nq = max(0, min(cw, d - n0)) >> 2;          // quads of columns here
    float *sq = reinterpret_cast<float *>(lds);           // [rows][cw/4]
    const float *gain = md.g_attn + (size_t)a.layer_begin * d;
    for (int it = tid; it < rows * nq; it += WG_THREADS) {
        int m = it / nq, c = n0 + (it - m * nq) * 4;
        int tok = row_token(a, m);
        const uint16_t *src = tok >= 0 ? md.emb + (size_t)tok * d + c : a.pf_emb + (size_t)m * d + c;
        uint2 r = *reinterpret_cast<const uint2 *>(src);
        float v[4] = {__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u), __uint_as_float(r.y << 16),
                      __uint_as_float(r.y & 0xFFFF0000u)};
        *reinterpret_cast<float4 *>(a.sc.h + (size_t)m * d + c) = make_float4(v[0], v[1], v[2], v[3]);
        sq[it] = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
        float4 g = *reinterpret_cast<const float4 *>(gain + c);
        float x[4] = {v[0] * g.x, v[1] * g.y, v[2] * g.z, v[3] * g.w};
        store_split4(a.sc.xn, rows, m, c, x);
    }
    __syncthreads();
    if (tid < rows) {
        float t = 0.f;
        for (int j = 0; j < nq; ++j) t += sq[tid * nq + j];
        store_dev32(a.sc.ss_a + (size_t)blockIdx.x * md.rows_max + tid, t);
    }
}

// ------------------------------------------------------------------ attention

constexpr float ATT_NEG = -1.0e30f;  // finite stand-in for "no position seen yet"

__device__ __forceinline__ uint2 load_global8(const void *p)
{
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
    u32x2_t v = *as_global(reinterpret_cast<const u32x2_t *>(p));
    return make_uint2(v[0], v[1]);
}

typedef __attribute__((ext_vector_type(4))) short s16x4_t;

__device__ __forceinline__ bf16x8_t pack_bf16x8(const uint32_t *h)
{
    return __builtin_bit_cast(bf16x8_t, make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)));
}

// Work item = (session, head, chunk of up to ATT_ROWS = 16 query rows, split of the cache's
// pages); the host picks the number of splits so that the items cover the chip and no wave
// gets more than ATT_TILES pages.  A wave takes whole pages (16 positions), page
// pg_lo + wave + t * WAVES being its tile t, and runs both products on the matrix cores:
//   scores  S[pos][row] = K . q^T   v_mfma_f32_16x16x32_bf16, A = 16 cached positions x 32
//           values straight from the page (lane l: position l & 15, values (l >> 4) * 8 ..),
//           B = the rows' q; three MFMAs per 32 values (k_hi q_hi + k_lo q_hi + k_hi q_lo);
//   output  O[row][dim] = p . V     v_mfma_f32_16x16x16bf16_1k, A = p in the layout the score
//           MFMA left it in (lane l: row l & 15, positions (l >> 4) * 4 ..), B = V, which the
//           cache stores transposed inside a page ([term][dim][position]) so that a lane's
//           four positions are 8 contiguous bytes; p and V as two bf16 terms, three MFMAs.
// All of a wave's score tiles stay in registers, so the softmax is two-pass inside the wave
// (no rescaling).  q and the cached k use the same pair-interleaved order inside a head, so
// their dot product is unchanged.  The waves' un-normalised results (accumulator, max, sum)
// are merged through LDS in wave order.  With one split the normalised output is written
// directly; otherwise every item writes its partial and counts itself in the unit's counter,
// and the item that arrives last merges the unit's partials in split order (the result does
// not depend on arrival order) and clears the counter for the next launch.  Nothing waits.
template <int HD>
__device__ void att_stage(const PassArgs &a, int layer, char *lds)
{
    constexpr int KT = HD / 32;  // 32-value steps of a score
    constexpr int NT = HD / 16;  // 16-column tiles of the output
    constexpr int REC = HD + 2;
    const int H = a.H, d = a.d, Kpad_d = a.Kpad_d, M = a.M;  // copies in the launch arguments: no load before the first address
    const int n_chunks = (M + ATT_ROWS - 1) / ATT_ROWS;
    const int n_splits = a.att_splits;
    const int n_items = a.n_sess * H * n_chunks * n_splits;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lm = lane & 15, quad = lane >> 4;
    float *wbuf = reinterpret_cast<float *>(lds);  // [WAVES][ATT_ROWS][REC]
    int *lastf = reinterpret_cast<int *>(wbuf + (size_t)WAVES * ATT_ROWS * REC);
    const size_t rec_page = (size_t)KV_PAGE * 2 * HD;  // elements of one (page, head) record

    trace_stamp(a, 0, 0);
    for (int item = blockIdx.x; item < n_items; item += a.nwg) {
        int unit = item / n_splits, sp = item - unit * n_splits;
        int s = unit / (H * n_chunks), rem = unit - s * (H * n_chunks);
        int hh = rem / n_chunks, ch = rem - hh * n_chunks;
        int r0 = ch * ATT_ROWS, nr = min(ATT_ROWS, M - r0);
        // session 0's descriptor also travels by value in the launch arguments: no dependent load
        const int *page_table = EE_SESS(a, s, page_table);
        const uint16_t *kpool = EE_SESS(a, s, kpool);
        const uint16_t *vpool = EE_SESS(a, s, vpool);
        const int n_pages = EE_SESS(a, s, n_pages);
        const int P = a.mode == 1 ? a.pf_pos0 : EE_SESS(a, s, kv_len);  // position of the first row
        const int n_pos = P + r0 + nr;  // positions visible to the chunk's last row
        const int n_pg = (n_pos + KV_PAGE - 1) / KV_PAGE;
        const int pg_lo = n_pg * sp / n_splits, pg_hi = n_pg * (sp + 1) / n_splits;
        const int T = max(0, (pg_hi - pg_lo - wave + WAVES - 1) / WAVES);  // tiles of this wave, <= ATT_TILES
        const int cbase = EE_SESS(a, s, contig_base);
        int my_pg = 0;  // physical page of this wave's tile number `lane`
        if (cbase >= 0)
            my_pg = cbase + pg_lo + wave + lane * WAVES;  // consecutive pages: no lookup, K can be requested together with q
        else if (lane < T)
            my_pg = as_global(page_table)[pg_lo + wave + lane * WAVES];

        // Requests first, uses after: the rows' q and the K of the wave's first tile (most waves
        // have one tile) travel together; with consecutive pages nothing had to be loaded to
        // know where K is.
        const int mrow = min(lm, nr - 1);
        f32x4_t qraw[KT][2];
        {
            const float *qp = a.sc.q + (size_t)(s * M + r0 + mrow) * d + hh * HD + quad * 8;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                qraw[kt][0] = *as_global(reinterpret_cast<const f32x4_t *>(qp + kt * 32));
                qraw[kt][1] = *as_global(reinterpret_cast<const f32x4_t *>(qp + kt * 32 + 4));
            }
        }
        uint4 k0h[KT], k0l[KT];
        if (T > 0) {
            const int page = __builtin_amdgcn_readlane(my_pg, 0);
            const uint16_t *kb = kpool + (((size_t)layer * n_pages + page) * H + hh) * rec_page + (size_t)lm * (2 * HD) + quad * 8;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                k0h[kt] = load_global16(kb + kt * 32);
                k0l[kt] = load_global16(kb + HD + kt * 32);
            }
        }
        // q as MFMA B operands, two bf16 terms (rows past the chunk repeat its last row)
        bf16x8_t qh[KT], ql[KT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            uint32_t h[8], l[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                split_bf16(qraw[kt][0][e], h[e], l[e]);
                split_bf16(qraw[kt][1][e], h[4 + e], l[4 + e]);
            }
            qh[kt] = pack_bf16x8(h);
            ql[kt] = pack_bf16x8(l);
        }
        // pass 1: score tiles
        f32x4_t S[ATT_TILES];
        const int last_pos = P + r0 + mrow;  // last position this lane's row may see
#pragma unroll
        for (int t = 0; t < ATT_TILES; ++t) {
            S[t] = (f32x4_t){ATT_NEG, ATT_NEG, ATT_NEG, ATT_NEG};
            if (t < T) {
                const int page = __builtin_amdgcn_readlane(my_pg, t);
                const uint16_t *kb = kpool + (((size_t)layer * n_pages + page) * H + hh) * rec_page + (size_t)lm * (2 * HD) + quad * 8;
                uint4 kh[KT], kl[KT];
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    kh[kt] = t == 0 ? k0h[kt] : load_global16(kb + kt * 32);
                    kl[kt] = t == 0 ? k0l[kt] : load_global16(kb + HD + kt * 32);
                }
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    const bf16x8_t Ah = __builtin_bit_cast(bf16x8_t, kh[kt]), Al = __builtin_bit_cast(bf16x8_t, kl[kt]);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Ah, qh[kt], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Al, qh[kt], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Ah, ql[kt], acc, 0, 0, 0);
                }
                const int pos0 = (pg_lo + wave + t * WAVES) * KV_PAGE + quad * 4;
#pragma unroll
                for (int r = 0; r < 4; ++r) S[t][r] = pos0 + r <= last_pos ? acc[r] * a.att_scale : ATT_NEG;
            }
        }
        if (a.sc.trace) trace_stamp(a, 0, 1);
        float mx = ATT_NEG;
#pragma unroll
        for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, S[t][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));

        // pass 2: probabilities and output tiles
        f32x4_t O[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) O[nt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        float lsum = 0.f;
#pragma unroll
        for (int t = 0; t < ATT_TILES; ++t) {
            if (t < T) {
                const int page = __builtin_amdgcn_readlane(my_pg, t);
                const uint16_t *vb = vpool + (((size_t)layer * n_pages + page) * H + hh) * rec_page + (size_t)lm * KV_PAGE + quad * 4;
                uint2 vh[NT], vl[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    vh[nt] = load_global8(vb + (size_t)(nt * 16) * KV_PAGE);
                    vl[nt] = load_global8(vb + (size_t)(HD + nt * 16) * KV_PAGE);
                }
                uint32_t ph[4], pl[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float pr = S[t][r] > 0.5f * ATT_NEG ? __expf(S[t][r] - mx) : 0.f;
                    lsum += pr;
                    split_bf16(pr, ph[r], pl[r]);
                }
                const s16x4_t Ph = __builtin_bit_cast(s16x4_t, make_uint2(ph[0] | (ph[1] << 16), ph[2] | (ph[3] << 16)));
                const s16x4_t Pl = __builtin_bit_cast(s16x4_t, make_uint2(pl[0] | (pl[1] << 16), pl[2] | (pl[3] << 16)));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const s16x4_t Vh = __builtin_bit_cast(s16x4_t, vh[nt]), Vl = __builtin_bit_cast(s16x4_t, vl[nt]);
                    O[nt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(Ph, Vh, O[nt], 0, 0, 0);
                    O[nt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(Pl, Vh, O[nt], 0, 0, 0);
                    O[nt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(Ph, Vl, O[nt], 0, 0, 0);
                }
            }
        }
        lsum += __shfl_xor(lsum, 16, 64);
        lsum += __shfl_xor(lsum, 32, 64);
        // this wave's record: lane holds O[row quad*4 + r][column nt*16 + lm]; max and sum per row lm
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (quad * 4 + r < nr) wbuf[((size_t)wave * ATT_ROWS + quad * 4 + r) * REC + nt * 16 + lm] = O[nt][r];
        if (quad == 0 && lm < nr) {
            float *w = wbuf + ((size_t)wave * ATT_ROWS + lm) * REC;
            w[HD] = mx;
            w[HD + 1] = lsum;
        }
        __syncthreads();
        trace_stamp(a, 0, 2);
        // merge the waves, fixed order
        if (n_splits == 1) {
            for (int t = tid; t < nr * HD; t += WG_THREADS) {
                int i = t / HD, e = t - i * HD;
                float gm = ATT_NEG;
                for (int w = 0; w < WAVES; ++w) gm = fmaxf(gm, wbuf[((size_t)w * ATT_ROWS + i) * REC + HD]);
                float num = 0.f, den = 0.f;
                for (int w = 0; w < WAVES; ++w) {
                    const float *wr = wbuf + ((size_t)w * ATT_ROWS + i) * REC;
                    float f = __expf(wr[HD] - gm);
                    num += wr[e] * f;
                    den += wr[HD + 1] * f;
                }
                uint32_t vh, vl;
                split_bf16(num / den, vh, vl);
                a.sc.attn[x_index(a.rows, s * M + r0 + i, hh * HD + e, 0)] = (uint16_t)vh;
                a.sc.attn[x_index(a.rows, s * M + r0 + i, hh * HD + e, 1)] = (uint16_t)vl;
            }
        } else {
            float *out = a.sc.att_part + (size_t)item * ATT_ROWS * REC;
            for (int t = tid; t < nr * REC; t += WG_THREADS) {
                int i = t / REC, e = t - i * REC;
                float gm = ATT_NEG;
                for (int w = 0; w < WAVES; ++w) gm = fmaxf(gm, wbuf[((size_t)w * ATT_ROWS + i) * REC + HD]);
                float r;
                if (e == HD) {
                    r = gm;
                } else {
                    r = 0.f;
                    for (int w = 0; w < WAVES; ++w) {
                        const float *wr = wbuf + ((size_t)w * ATT_ROWS + i) * REC;
                        r += wr[e] * __expf(wr[HD] - gm);
                    }
                }
                store_dev32(out + (size_t)i * REC + e, r);
            }
            trace_stamp(a, 0, 3);
            wait_vmem();      // this item's partials are visible device-wide ...
            __syncthreads();  // ... for every wave, before it is counted
            if (tid == 0) {
                int before = __hip_atomic_fetch_add(a.sc.att_count + unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *lastf = before == n_splits - 1 ? 1 : 0;
            }
            __syncthreads();
            trace_stamp(a, 0, 4);
            if (*lastf) {
                const float *base = a.sc.att_part + (size_t)unit * n_splits * ATT_ROWS * REC;
                const size_t sp_stride = (size_t)ATT_ROWS * REC;
                for (int t = tid; t < nr * HD; t += WG_THREADS) {
                    int i = t / HD, e = t - i * HD;
                    const float *row = base + (size_t)i * REC;
                    // all loads first, so that they are in flight together
                    float pm[ATT_MAX_SPLITS], pv[ATT_MAX_SPLITS], pl[ATT_MAX_SPLITS];
#pragma unroll
                    for (int k = 0; k < ATT_MAX_SPLITS; ++k) {
                        const float *r = row + min(k, n_splits - 1) * sp_stride;
                        pm[k] = load_dev32(r + HD);
                        pv[k] = load_dev32(r + e);
                        pl[k] = load_dev32(r + HD + 1);
                    }
                    float gm = ATT_NEG;
#pragma unroll
                    for (int k = 0; k < ATT_MAX_SPLITS; ++k)
                        if (k < n_splits) gm = fmaxf(gm, pm[k]);
                    float num = 0.f, den = 0.f;
#pragma unroll
                    for (int k = 0; k < ATT_MAX_SPLITS; ++k)
                        if (k < n_splits) {
                            float f = __expf(pm[k] - gm);
                            num += pv[k] * f;
                            den += pl[k] * f;
                        }
                    uint32_t vh, vl;
                    split_bf16(num / den, vh, vl);
                    a.sc.attn[x_index(a.rows, s * M + r0 + i, hh * HD + e, 0)] = (uint16_t)vh;
                    a.sc.attn[x_index(a.rows, s * M + r0 + i, hh * HD + e, 1)] = (uint16_t)vl;
                }
                if (tid == 0) __hip_atomic_store(a.sc.att_count + unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
        trace_stamp(a, 0, 5);
    }
}

// ------------------------------------------------------------------ accept

__device__ __forceinline__ int2 load_cand(const int2 *p)
{
    const unsigned long long v = __hip_atomic_load(as_global(reinterpret_cast<const unsigned long long *>(p)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_int2((int)(unsigned)v, (int)(unsigned)(v >> 32));
}

// One workgroup: global argmax per row, confidence, accept rule per session, publication.
// Reads the candidates with device scope: they may have been written earlier in this launch.
__device__ void accept_stage(const PassArgs &a, char *lds)
{
    const ModelDev &md = a.mdv;
    const int rows = a.rows, M = a.M;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int *tok = reinterpret_cast<int *>(lds);
    float *conf = reinterpret_cast<float *>(lds) + EE_MAX_ROWS;
    for (int m = wave; m < rows; m += WAVES) {
        float bv = -INFINITY;
        int bi = 0x7FFFFFFF;
        for (int g = lane; g < a.nwg; g += 64) {
            int2 c = load_cand(a.sc.cand + (size_t)g * md.rows_max + m);
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
        // confidence (paper Eq. 4): max softmax = 1 / sum_j exp(z_j - z_max), from the
        // workgroups' sums, each rescaled from its own maximum to the global one
        float se = 0.f;
        for (int g = lane; g < a.nwg; g += 64) {
            const float vg = __int_as_float(load_cand(a.sc.cand + (size_t)g * md.rows_max + m).x);
            const float sg = load_dev32(a.sc.cand_sum + (size_t)g * md.rows_max + m);
            if (sg > 0.f) se += sg * __expf(vg - bv);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) se += __shfl_xor(se, off, 64);
        if (lane == 0) {
            tok[m] = bi;
            conf[m] = 1.0f / se;
        }
    }
    __syncthreads();
    const int s = threadIdx.x;
    if (s < a.n_sess) {
        const SessDev &sd = a.sess[s];
        ee_verify_result *res = sd.result;
        const int *t = tok + s * M;
        const float *cf = conf + s * M;
        int dev_err = __hip_atomic_load(a.sc.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (a.head_kind == HEAD_PREFILL) {
            int last = t[M - 1];
            res->next_token = last;
            res->device_status = dev_err;
            sd.state[1] = last;
        } else {
            const int gamma = M - 1;
            int dr[EE_MAX_M];
#pragma unroll
            for (int i = 0; i < EE_MAX_M - 1; ++i) dr[i] = i < gamma ? sd.drafts[i] : -1;
            int delta = 0;
#pragma unroll
            for (int i = 0; i < EE_MAX_M - 1; ++i)
                if (delta == i && i < gamma && dr[i] == t[i]) delta = i + 1;
            if (a.head_kind == HEAD_EXIT) {
                for (int i = 0; i < M; ++i) {
                    res->exit_tokens[a.head_idx][i] = t[i];
                    res->exit_conf[a.head_idx][i] = cf[i];
                }
                res->exit_accept_len[a.head_idx] = delta;
            } else {
                for (int i = 0; i < M; ++i) {
                    res->final_tokens[i] = t[i];
                    res->final_conf[i] = cf[i];
                }
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

// ------------------------------------------------------------------ kernels of the pass
//
// Stage list of a segment: [EMBED] { QKV ATT O GU DN } x layers [HEAD ACCEPT].
// Consecutive GEMM stages run inside one launch of the chain kernel with a grid barrier
// between them; attention, embedding and accept are launches of their own.

struct StageDesc {
    int type, kind, layer;
};

__device__ __forceinline__ StageDesc stage_decode(const PassArgs &a, int ph)
{
    StageDesc sd = {ST_NONE, 0, 0};
    const int per_layer = 5;
    int idx = ph - (a.do_embed ? 1 : 0);
    if (idx < 0) {
        sd.type = ST_EMBED;
        return sd;
    }
    const int nl = a.layer_end - a.layer_begin;
    if (idx < per_layer * nl) {
        int li = idx / per_layer, r = idx - li * per_layer;
        sd.layer = a.layer_begin + li;
        if (r == 0) {
            sd.type = ST_GEMM;
            sd.kind = G_QKV;
        } else if (r == 1) {
            sd.type = ST_ATT;
        } else {
            sd.type = ST_GEMM;
            sd.kind = G_O + (r - 2);
        }
        return sd;
    }
    idx -= per_layer * nl;
    if (a.head_kind != HEAD_NONE) {
        if (idx == 0) {
            sd.type = ST_GEMM;
            sd.kind = G_HEAD;
        } else if (idx == 1) {
            sd.type = ST_ACCEPT;
        }
    }
    return sd;
}

__device__ __forceinline__ GemmIn gemm_input(const PassArgs &a, int kind)
{
    const ModelDev &md = a.mdv;
    switch (kind) {
    case G_QKV: return GemmIn{a.sc.xn, a.sc.ss_a};
    case G_O: return GemmIn{a.sc.attn, nullptr};
    case G_GU: return GemmIn{a.sc.xn, a.sc.ss_f};
    case G_DN: return GemmIn{a.sc.u, nullptr};
    default: return GemmIn{a.sc.xh, a.sc.ss_a};
    }
}

__device__ __forceinline__ GemmEpi gemm_epi(const PassArgs &a, int kind, int layer)
{
    const ModelDev &md = a.mdv;
    GemmEpi ep = {nullptr, nullptr, nullptr};
    if (kind == G_O) {
        ep.gain_xn = md.g_ffn + (size_t)layer * md.d;
        ep.ss_out = a.sc.ss_f;
    } else if (kind == G_DN) {
        if (layer + 1 < md.L) ep.gain_xn = md.g_attn + (size_t)(layer + 1) * md.d;
        if (layer + 1 == a.layer_end && a.head_kind != HEAD_NONE) ep.gain_xh = a.head_gain;
        ep.ss_out = a.sc.ss_a;
    }
    return ep;
}

// GEMM stages [ph_lo, ph_hi) of the stage list (all of them must be GEMM stages).
// MT = 16-row tiles of the pass (rows <= 16 * MT).
template <int MT>
__global__ void __launch_bounds__(WG_THREADS) ee_gemm_chain_kernel(PassArgs a_by_value)
{
    extern __shared__ __align__(16) char lds[];
    const PassArgs &a = warmed_arguments();
    // The tables indexed by the stage kind are read from the descriptor in device memory; the
    // first stage's entries (the only ones of a one-stage launch) come with the launch
    // arguments, so that nothing has to be loaded before the first weight address is known.
    const ModelDev *mdp = a.md;
    unsigned nbar = 0;
    if (a.mode == 2) {  // measurement aid: layer_end grid barriers and nothing else
        for (int i = 0; i < a.layer_end; ++i)
            grid_barrier(a.sc.bar_flags, a.nwg, a.epoch_base + (++nbar), a.sc.err, a.spin_limit);
        return;
    }
    trace_stamp_wg(a, 0);
    uint4 buf[D];           // weight tiles in flight; carried from one stage into the next
    bool have_pre = false;  // buf holds the first tiles of the coming stage
    for (int ph = a.ph_lo; ph < a.ph_hi; ++ph) {
        if (ph > a.ph_lo) {
            wait_vmem();
            trace_stamp(a, ph - a.ph_lo - 1, 7);
            grid_barrier(a.sc.bar_flags, a.nwg, a.epoch_base + (++nbar), a.sc.err, a.spin_limit);
        }
        const StageDesc st = stage_decode(a, ph);
        NextGemm nx = {nullptr, nullptr};
        if (ph + 1 < a.ph_hi) {
            const StageDesc sn = stage_decode(a, ph + 1);
            nx.pl = &mdp->plan[sn.kind];
            nx.W = mdp->w[sn.kind] + (size_t)sn.layer * mdp->wstride[sn.kind];
        }
        const GemmIn in = gemm_input(a, st.kind);
        const GemmEpi ep = gemm_epi(a, st.kind, st.layer);
        if (ph == a.ph_lo)
            gemm_stage_t<MT>(a, st.kind, st.layer, a.plan0, a.W0, in, ep, buf, have_pre, nx, lds, 0);
        else
            gemm_stage_t<MT>(a, st.kind, st.layer, mdp->plan[st.kind], mdp->w[st.kind] + (size_t)st.layer * mdp->wstride[st.kind],
                             in, ep, buf, have_pre, nx, lds, ph - a.ph_lo);
        trace_stamp(a, ph - a.ph_lo, 6);
    }
    if (a.fuse_accept) {
        // The launch ended with a head stage: the workgroup whose candidates arrive last also
        // runs the accept step (one launch less per head); the counter is left at zero.
        int *lastf = reinterpret_cast<int *>(lds + 8192);
        wait_vmem();      // this workgroup's candidates are visible device-wide ...
        __syncthreads();  // ... for every wave, before it is counted
        if (threadIdx.x == 0) {
            const int before = __hip_atomic_fetch_add(a.sc.head_count, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *lastf = before == a.nwg - 1 ? 1 : 0;
            if (*lastf) __hip_atomic_store(a.sc.head_count, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (*lastf) accept_stage(a, lds);
    }
    trace_stamp_wg(a, 1);
}

template <int HD>
__global__ void __launch_bounds__(WG_THREADS) ee_att_kernel(PassArgs a_by_value)
{
    extern __shared__ __align__(16) char lds[];
    const PassArgs &a = warmed_arguments();
    trace_stamp_wg(a, 0);
    att_stage<HD>(a, stage_decode(a, a.ph_lo).layer, lds);
    trace_stamp_wg(a, 1);
}

// embedding, accept: stage ph_lo
__global__ void __launch_bounds__(WG_THREADS) ee_misc_kernel(PassArgs a_by_value)
{
    extern __shared__ __align__(16) char lds[];
    const PassArgs &a = warmed_arguments();
    const StageDesc st = stage_decode(a, a.ph_lo);
    trace_stamp_wg(a, 0);
    if (st.type == ST_EMBED)
        embed_stage(a, lds);
    else if (st.type == ST_ACCEPT && blockIdx.x == 0)
        accept_stage(a, lds);
    trace_stamp_wg(a, 1);
}

// ------------------------------------------------------------------ load-time kernels

// source row of output column n for the row orders the stages expect
__device__ __forceinline__ int perm_row(int perm, int n, int d, int hd, int F)
{
    if (perm == PERM_QKV) {
        int sect = n / d, c = n - sect * d;
        if (sect >= 2) return n;
        int head = c / hd, e = c - head * hd;
        int src_e = (e & 1) ? (e >> 1) + (hd >> 1) : (e >> 1);  // RoPE pair (j, j+hd/2) -> columns (2j, 2j+1)
        return sect * d + head * hd + src_e;
    }
    if (perm == PERM_GU) {
        int tile = n >> 4, r = n & 15;
        int p = tile >> 1, which = tile & 1;                     // gate tile p, up tile p, gate tile p+1, ...
        return which * F + p * 16 + r;
    }
    return n;
}

// row-major bf16 src[N][K] -> the tiled layout of GemmPlan; block g writes workgroup g's tiles,
// sub-wave `sub` of the block those of wave w = sub, sub + nsub, ...
__global__ void tile_weights_kernel(const uint16_t *__restrict__ src, uint4 *__restrict__ dst, GemmPlan pl, int nwg,
                                    int perm, int d, int hd, int F)
{
    const int g = blockIdx.x;
    int nt0, n_local;
    wg_units(pl, nwg, g, nt0, n_local);
    if (n_local == 0) return;
    const int lane = threadIdx.x & 63, sub = threadIdx.x >> 6, nsub = blockDim.x >> 6;
    const int n_groups = (n_local + pl.GRP - 1) / pl.GRP;
    for (int w = sub; w < WAVES; w += nsub) {
        int step = 0;
        for (int gi = 0; gi < n_groups; ++gi) {
            for (int kb = 0; kb < pl.nKB; ++kb) {
                const Seg s = seg_setup(pl, nt0, n_local, w, gi, kb);
                for (int ntg = 0; ntg < s.gn; ++ntg) {
                    for (int kk = 0; kk < s.slen; ++kk, ++step) {
                        int n = (nt0 + gi * pl.GRP + ntg) * 16 + (lane & 15);
                        int k0 = (s.kst + s.s0 + kk) * 32 + (lane >> 4) * 8;
                        uint16_t v[8];
                        int row = n < pl.N ? perm_row(perm, n, d, hd, F) : -1;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            int k = k0 + e;
                            v[e] = (row >= 0 && k < pl.K) ? src[(size_t)row * pl.K + k] : (uint16_t)0;
                        }
                        uint4 o;
                        o.x = v[0] | ((uint32_t)v[1] << 16);
                        o.y = v[2] | ((uint32_t)v[3] << 16);
                        o.z = v[4] | ((uint32_t)v[5] << 16);
                        o.w = v[6] | ((uint32_t)v[7] << 16);
                        dst[((size_t)((size_t)step * nwg + g) * WAVES + w) * 64 + lane] = o;
                    }
                }
            }
        }
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

// plain copy of n 16-byte words: the reference for what the HBM traffic counters read per byte
__global__ void __launch_bounds__(256) ee_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

// the same for v_mfma_f32_16x16x16bf16_1k: A[i][k] from lane (i + 16*(k/4)) element k%4,
// B[k][j] likewise with j, D as above
__global__ void mfma16_layout_probe_kernel(const uint2 *a, const uint2 *b, float *out)
{
    s16x4_t A = __builtin_bit_cast(s16x4_t, a[threadIdx.x]);
    s16x4_t B = __builtin_bit_cast(s16x4_t, b[threadIdx.x]);
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(A, B, acc, 0, 0, 0);
    for (int r = 0; r < 4; ++r) out[threadIdx.x * 4 + r] = acc[r];
}

}  // namespace ee
