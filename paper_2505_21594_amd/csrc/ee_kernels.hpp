// gfx950 kernels of the verification pass.
//
// A segment of the pass (embedding, a range of layers, optionally an LM head with its
// accept step) is a list of stages, one launch each.  Per layer (Eq. 3 of the paper,
// f = Llama-2 block) there are five:
//   QKV   x_hat . [Wq;Wk;Wv]^T, * rstd, RoPE, q -> scratch, k/v -> paged bf16 cache
//   ATT   causal attention of the new rows over the cache         -> attn
//   O     h += attn . Wo^T
//   GU    u = silu(rstd * x_hat.Wg^T) * (rstd * x_hat.Wu^T)
//   DN    h += u . Wd^T
// Head (z^(l) = LMHead(h^(l)); accept rule of Eq. 2 / Eq. 5; confidence of Eq. 4):
//   HEAD    x_hat . W_lm^T, * rstd, argmax candidate and softmax denominator per workgroup
//   ACCEPT  global argmax (lowest id wins ties), confidence, accept length, publication
//           to pinned host memory, KV commit (run by the head launch's last workgroup).
// Kernels: ee_gemm_kernel<MT> for the five GEMM kinds (MT = 16-row tiles of the pass, rows <= 48),
// ee_att_kernel, ee_misc_kernel (embedding).
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

// Pointers read from descriptors in memory are generic to the compiler, and generic loads go
// through the flat path, whose completion also counts against the LDS counter: a wait for an
// LDS read would then drain every weight load in flight.  These helpers state that the
// address is global memory.
#define EE_GLOBAL __attribute__((address_space(1)))
#define EE_LDS __attribute__((address_space(3)))
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
__device__ __forceinline__ WRes buffer_resource(const void *p) { return weight_resource(reinterpret_cast<const uint4 *>(p)); }
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

// Device-scope accesses for the small buffers that one launch's workgroups exchange among
// themselves (attention partials of a split position range, argmax candidates of a head):
// stores write through to memory and loads bypass the per-XCD L2.  Everything else is read-only
// in a launch or crosses a kernel boundary.
__device__ __forceinline__ void store_dev64(void *p, uint2 v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), ((unsigned long long)v.y << 32) | v.x,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_dev32(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// the same for 16 bytes at byte offset `off` of a buffer (weight_resource): device-scope cache policy (sc1)
constexpr int CACHE_POLICY_DEVICE = 16;
__device__ __forceinline__ void store_dev128(WRes r, int off, float4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128((u32x4_t){__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)},
                                           r, off, 0, CACHE_POLICY_DEVICE);
}
__device__ __forceinline__ float4 load_dev128(WRes r, int off)
{
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, CACHE_POLICY_DEVICE);
    return make_float4(__uint_as_float(v[0]), __uint_as_float(v[1]), __uint_as_float(v[2]), __uint_as_float(v[3]));
}
__device__ __forceinline__ float load_dev32(const float *p)
{
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The value itself, but opaque to the optimiser: keeps per-thread index arithmetic of a stage
// from being hoisted to the kernel's start, where it would occupy registers throughout.
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
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
// at most n vector memory operations of this wave are still pending (n is rounded down to a
// value with an instruction of its own, which only makes the wait stricter)
__device__ __forceinline__ void wait_vmem_pending(int n)
{
#define EE_WAIT_CASE(N) case N: __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14)); break;
    switch (min(n, 31)) {
        EE_WAIT_CASE(0) EE_WAIT_CASE(1) EE_WAIT_CASE(2) EE_WAIT_CASE(3) EE_WAIT_CASE(4) EE_WAIT_CASE(5) EE_WAIT_CASE(6) EE_WAIT_CASE(7)
        EE_WAIT_CASE(8) EE_WAIT_CASE(9) EE_WAIT_CASE(10) EE_WAIT_CASE(11) EE_WAIT_CASE(12) EE_WAIT_CASE(13) EE_WAIT_CASE(14) EE_WAIT_CASE(15)
        EE_WAIT_CASE(16) EE_WAIT_CASE(17) EE_WAIT_CASE(18) EE_WAIT_CASE(19) EE_WAIT_CASE(20) EE_WAIT_CASE(21) EE_WAIT_CASE(22) EE_WAIT_CASE(23)
        EE_WAIT_CASE(24) EE_WAIT_CASE(25) EE_WAIT_CASE(26) EE_WAIT_CASE(27) EE_WAIT_CASE(28) EE_WAIT_CASE(29) EE_WAIT_CASE(30) EE_WAIT_CASE(31)
    }
#undef EE_WAIT_CASE
    asm volatile("" ::: "memory");
}
// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every
// vector memory operation of the wave, i.e. for all weight tiles a streaming wave has in
// flight; nothing that crosses these barriers goes through global memory.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
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
    int s = div_small(r, a.M);
    return EE_SESS(a, s, kv_len) + (r - s * a.M);
}

__device__ __forceinline__ int row_token(const PassArgs &a, int r)
{
    if (a.mode == 1) return a.pf_tokens[r];
    int s = div_small(r, a.M), i = r - s * a.M;
    return i == 0 ? EE_SESS(a, s, pending) : EE_SESS(a, s, drafts)[i - 1];
}

// ------------------------------------------------------------------ LDS map

struct Misc {  // views into the misc region of the LDS block
    float *rstd;       // [rows]
    float *rowss;      // [rows]  this workgroup's sum of h^2 per row (O / DN stages)
    int *pos;          // [rows]
    long long *kvoff;  // [rows]  element offset of the row's (layer, page, head 0) record in the KV pools
    float *bestv;      // [rows]
    int *besti;        // [rows]
    float *sume;       // [rows]  sum of exp(logit - bestv) over the columns seen so far
    int *lastf;        // "this workgroup finished the head launch last"
};

constexpr int MISC_BYTES = EE_MAX_ROWS * (8 + 6 * 4) + 64;

__device__ __forceinline__ Misc misc_views(const StageLds &ly, char *lds)
{
    Misc m;
    char *p = lds + ly.misc_off;
    const int R = EE_MAX_ROWS;
    m.kvoff = reinterpret_cast<long long *>(p);
    p += (size_t)R * 8;
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
    p += (size_t)R * 4;
    m.lastf = reinterpret_cast<int *>(p);
    return m;
}

// ------------------------------------------------------------------ weight-stream geometry

__device__ __host__ inline void wg_units(const GemmPlan &pl, int g, int &nt0, int &n_local)
{
    int u0 = 0, u1 = 0;
    if (g < pl.nwg) unit_range(pl.U, pl.nwg >> pl.ksl, g >> pl.ksl, u0, u1);  // workgroups past the stage's count own nothing
    nt0 = u0 * pl.tpu;
    n_local = (u1 - u0) * pl.tpu;
}

// k-steps of streaming wave w: its k-tiles are w, w + SWAVES, ...
__device__ __host__ inline int wave_ksteps(int KT, int w) { return KT > w ? (KT - w + SWAVES - 1) / SWAVES : 0; }

// ------------------------------------------------------------------ GEMM stage

struct GemmIn {
    const uint16_t *x;  // the input (already scaled by the norm gain) as two bf16 terms, k-tile-major (x_index)
    const float *ss;    // [nwg][rows_max] partial sums of squares for rstd, or nullptr
};

// GEMM inputs are stored the way the stages consume them: [k-tile][term][row][32] bf16 with
// `rows` = the rows of this pass, term 0 = hi, 1 = lo.  A range of k-tiles (all rows, both
// terms) is then one contiguous range, which 1 KB loads copy straight into LDS, and the 16 rows x
// 4 quads of one MFMA operand read one contiguous kilobyte of LDS.
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
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
    *reinterpret_cast<EE_GLOBAL u32x2_t *>(as_global_mut(x) + x_index(rows, m, k, 0)) = (u32x2_t){h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
    *reinterpret_cast<EE_GLOBAL u32x2_t *>(as_global_mut(x) + x_index(rows, m, k, 1)) = (u32x2_t){l[0] | (l[1] << 16), l[2] | (l[3] << 16)};
}

// Helper waves: copy k-tiles [kt0, kt0 + klen) of the input (all rows, both terms: one
// contiguous range in memory) straight into LDS at dst.  One load instruction moves 64 x 16
// bytes; no registers hold the data.  The caller waits (wait_vmem) before it tells the others.
__device__ __forceinline__ int stage_block(const uint16_t *x, int rows, int kt0, int klen, char *dst, int hwave, int lane)
{
    const size_t tile_elems = (size_t)2 * rows * 32;          // one k-tile: both terms, all rows
    const uint16_t *src = x + (size_t)kt0 * tile_elems;
    const int nchunk = klen * 2 * rows * 4;                     // 16-byte chunks of the block
    for (int c0 = hwave * 64; c0 < nchunk; c0 += HWAVES * 64)
        if (c0 + lane < nchunk)
            __builtin_amdgcn_global_load_lds((const EE_GLOBAL void *)(src + (size_t)(c0 + lane) * 8),
                                             (EE_LDS void *)(dst + (size_t)c0 * 16), 16, 0, 0);
    return nchunk > hwave * 64 ? (nchunk - hwave * 64 + HWAVES * 64 - 1) / (HWAVES * 64) : 0;  // load instructions of this wave
}

// rstd[m] = 1/sqrt(sum_g ss[g][m] / d + eps) into LDS, fixed summation order; helper waves only.
// Ordinary loads, which the XCD's L2 serves to all but the first workgroup: every workgroup
// reads the same few kilobytes.
__device__ __forceinline__ void load_rstd(const float *ss, int nwg, int rows_max, int rows, int d, float eps,
                                          float *rstd_lds, int hwave, int lane)
{
    for (int m = hwave; m < rows; m += HWAVES) {
        float v[4];                                              // at most 256 workgroups: all four requested together
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = lane + 64 * j < nwg ? *as_global(ss + (size_t)(lane + 64 * j) * rows_max + m) : 0.f;
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) s += v[j];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) rstd_lds[m] = 1.0f / sqrtf(s / (float)d + eps);
    }
}

__device__ __forceinline__ bool cand_better(float v, int i, float bv, int bi)
{
    return v > bv || (v == bv && i < bi);
}

struct GemmEpi {           // what the O / DN / AU epilogue produces besides h
    const float *gain_xn;  // gain of the next GEMM input (xn), or nullptr
    const float *gain_xh;  // gain of the LM-head input (xh, at the exit's head rows), or nullptr
    float *ss_out;         // [nwg][rows_max] partial sums of h^2, or nullptr
    float *ss_head;        // [nwg][rows_max] partial sums of squares of the LM-head input's rows (at the head rows), or nullptr
    const float *bias;     // AD / AU: bias per output column
    int xa_out;            // DN: also emit h itself as the adapters' input (xa)
};

// Epilogue of one chunk of gn n-tiles starting at n-tile nt_first: sum the nsum partial tiles in
// the slot buffer (the streaming waves', or the K splits' when K is split over workgroups; fixed
// order), apply the stage's element-wise tail.  All threads.
__device__ __forceinline__ void gemm_epilogue(const PassArgs &a, int kind, int layer, const StageLds &ly, int nt_first,
                                              int gn, int rows, const GemmEpi &ep, const Misc &mi, char *lds, const int nsum)
{
    const ModelDev &md = a.mdv;
    const float *slots = reinterpret_cast<const float *>(lds);
    const int tid = opaque(threadIdx.x);
    const size_t wstride = (size_t)ly.chunk * rows * 16;  // floats per wave in the slot buffer
    if (kind == G_GU) {
        const int items = (gn >> 1) * rows * 4;
        for (int idx = tid; idx < items; idx += WG_THREADS) {
            int p = div_small(idx, rows * 4), rem = idx - p * rows * 4;
            int m = rem >> 2, qd = rem & 3;
            const float *sg = slots + ((size_t)(2 * p) * rows + m) * 16 + qd * 4;
            const float *su = sg + (size_t)rows * 16;
            float4 G = make_float4(0.f, 0.f, 0.f, 0.f), U = G;
#pragma unroll 2
            for (int w = 0; w < nsum; ++w) {
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
    float *zbuf = reinterpret_cast<float *>(lds + ly.zbuf_off);  // head: [rows][chunk*16] logits of this chunk; O/DN: squares
    const int items = gn * rows * 4;
    for (int idx = tid; idx < items; idx += WG_THREADS) {
        int ntg = div_small(idx, rows * 4), rem = idx - ntg * rows * 4;
        int m = rem >> 2, qd = rem & 3;
        const int n = (nt_first + ntg) * 16 + qd * 4;  // four consecutive output columns
        // What the item reads from global memory is requested first, all of it at once: the sum of
        // the partial tiles below then runs while it is on its way (one after the other, after the
        // sum, these loads were two memory latencies at the end of every launch).
        f32x4_t g_a = (f32x4_t){0.f, 0.f, 0.f, 0.f}, g_b = g_a, g_c = g_a;
        int qkv_sect = 0, qkv_c = 0, qkv_head = 0, qkv_e = 0, qkv_ses = 0;
        if (kind == G_O || kind == G_DN || kind == G_AU) {
            if (n < md.d) {
                g_a = *as_global(reinterpret_cast<const f32x4_t *>(a.sc.h + (size_t)m * md.d + n));
                if (kind == G_AU) g_b = *as_global(reinterpret_cast<const f32x4_t *>(ep.bias + n));
                if (ep.gain_xn) g_b = *as_global(reinterpret_cast<const f32x4_t *>(ep.gain_xn + n));
                if (ep.gain_xh) g_c = *as_global(reinterpret_cast<const f32x4_t *>(ep.gain_xh + n));
            }
        } else if (kind == G_QKV) {
            qkv_sect = div_small(n, md.d);
            qkv_c = n - qkv_sect * md.d;
            qkv_head = div_small(qkv_c, md.hd);
            qkv_e = qkv_c - qkv_head * md.hd;
            qkv_ses = a.mode == 1 ? 0 : div_small(m, a.M);
            if (qkv_sect < 2)  // (cos, sin) of the row's position for the RoPE pairs of these four columns
                g_a = *as_global(reinterpret_cast<const f32x4_t *>(EE_SESS(a, qkv_ses, rope) + (size_t)mi.pos[m] * (md.hd >> 1) + (qkv_e >> 1)));
        } else if (kind == G_AD) {
            if (n < md.A) g_a = *as_global(reinterpret_cast<const f32x4_t *>(ep.bias + n));
        }
        const float *sp = slots + ((size_t)ntg * rows + m) * 16 + qd * 4;
        float4 S = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
        for (int w = 0; w < nsum; ++w) {
            float4 x = *reinterpret_cast<const float4 *>(sp + w * wstride);
            S.x += x.x; S.y += x.y; S.z += x.z; S.w += x.w;
        }
        if (kind == G_AD) {
            // hidden units of the exit head's adapters: silu(W_down . h + b_down)
            if (n < md.A) {
                const f32x4_t b = g_a;
                float pre[4] = {S.x + b[0], S.y + b[1], S.z + b[2], S.w + b[3]}, o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = pre[e] / (1.0f + __expf(-pre[e]));
                store_split4(a.sc.t, rows, m, n, o);
            }
        } else if (kind == G_O || kind == G_DN || kind == G_AU) {
            float sq = 0.f;
            if (n < md.d) {
                EE_GLOBAL f32x4_t *hp = reinterpret_cast<EE_GLOBAL f32x4_t *>(as_global_mut(a.sc.h) + (size_t)m * md.d + n);
                const f32x4_t hv = g_a;
                float v[4] = {hv[0] + S.x, hv[1] + S.y, hv[2] + S.z, hv[3] + S.w};
                if (kind == G_AU) {  // a side branch: a = h + W_up . t + b_up feeds the exit's LM head, h stays as it is
                    const f32x4_t b = g_b;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += b[e];
                } else {
                    *hp = (f32x4_t){v[0], v[1], v[2], v[3]};
                }
                if (ep.xa_out) store_split4(a.sc.xa, rows, m, n, v);
                sq = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                if (ep.gain_xn) {
                    const f32x4_t g = g_b;
                    float x[4] = {v[0] * g[0], v[1] * g[1], v[2] * g[2], v[3] * g[3]};
                    store_split4(a.sc.xn, rows, m, n, x);
                }
                if (ep.gain_xh) {
                    const f32x4_t g = g_c;
                    float x[4] = {v[0] * g[0], v[1] * g[1], v[2] * g[2], v[3] * g[3]};
                    store_split4(a.sc.xh, a.head_rows, a.head_row0 + m, n, x);
                }
            }
            zbuf[idx] = sq;  // (ntg, m, quad) order
        } else if (kind == G_QKV) {
            const int d = md.d, hd = md.hd;
            const float rs = mi.rstd[m];
            float v[4] = {S.x * rs, S.y * rs, S.z * rs, S.w * rs};
            const int sect = qkv_sect, c = qkv_c, head = qkv_head, e = qkv_e, ses = qkv_ses;
            if (sect < 2) {
                // columns are pair-interleaved inside a head: (e, e+1) = RoPE pair e/2
                const f32x4_t cs = g_a;
                float y0 = v[0] * cs[0] - v[1] * cs[1], y1 = v[1] * cs[0] + v[0] * cs[1];
                float y2 = v[2] * cs[2] - v[3] * cs[3], y3 = v[3] * cs[2] + v[2] * cs[3];
                v[0] = y0; v[1] = y1; v[2] = y2; v[3] = y3;
            }
            if (sect == 0) {
                *reinterpret_cast<EE_GLOBAL f32x4_t *>(as_global_mut(a.sc.q) + (size_t)m * d + c) = (f32x4_t){v[0], v[1], v[2], v[3]};
            } else {
                // cached value = hi + lo, two bf16 terms.  K: [position][term][hd]; V transposed
                // inside the page: [term][hd][position] (see the attention stage)
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
            float *zr = zbuf + (size_t)m * ly.chunk * 16 + ntg * 16 + qd * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (n + e >= md.V) z[e] = -INFINITY;
                zr[e] = z[e];
            }
            if (a.keep_logits) {
                const int per_head = a.n_sess * a.M, hj = m / per_head;  // the launch's rows: head after head
                EE_GLOBAL float *keep = as_global_mut(a.sc.logits) + ((size_t)(a.head_idx + hj) * md.rows_max + (m - hj * per_head)) * md.V;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n + e < md.V) keep[n + e] = z[e];
            }
        }
    }
    if (kind == G_O || kind == G_DN || kind == G_AU) {
        lds_barrier();
        if (tid < rows) {  // this chunk's sum of squares per row, fixed order
            float t = 0.f;
            for (int ntg = 0; ntg < gn; ++ntg)
                for (int qd = 0; qd < 4; ++qd) t += zbuf[(ntg * rows + tid) * 4 + qd];
            mi.rowss[tid] += t;
        }
    }
    if (kind == G_HEAD) {
        lds_barrier();
        const int lane = tid & 63, wave = tid >> 6;
        for (int m = wave; m < rows; m += WAVES) {
            float bv = -INFINITY;
            int bi = 0x7FFFFFFF;
            for (int c = lane; c < gn * 16; c += 64) {
                float z = zbuf[(size_t)m * ly.chunk * 16 + c];
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
            // sum of exp(z - bv) over the chunk's columns (masked columns hold -inf and add 0):
            // the softmax denominator for the confidence score (paper Eq. 4), kept relative to the
            // running maximum like the argmax candidate
            float se = 0.f;
            for (int c = lane; c < gn * 16; c += 64) se += __expf(zbuf[(size_t)m * ly.chunk * 16 + c] - bv);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) se += __shfl_xor(se, off, 64);
            if (lane == 0 && bv > -INFINITY) {  // (a chunk of masked columns only contributes nothing)
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

// K split over workgroups: instead of the epilogue, one chunk of gn n-tiles of this workgroup's
// partial sums (the streaming waves' tiles added up, fixed order) goes to memory, to
// part[split][n-tile][row][16].  All threads.
__device__ __forceinline__ void partial_store(const PassArgs &a, const GemmPlan &pl, const StageLds &ly, int nt_first, int gn,
                                              int rows, const char *lds)
{
    const float *slots = reinterpret_cast<const float *>(lds);
    const int tid = opaque(threadIdx.x);
    const size_t wstride = (size_t)ly.chunk * rows * 16;
    const int sp = blockIdx.x & ((1 << pl.ksl) - 1);
    const WRes out = buffer_resource(a.sc.part + ((size_t)sp * pl.NT + nt_first) * rows * 16);
    const int items = gn * rows * 4;            // (n-tile, row, quad of columns): the slot buffer's own order
    for (int idx = tid; idx < items; idx += WG_THREADS) {
        const float *p = slots + (size_t)idx * 4;
        float4 S = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
        for (int w = 0; w < SWAVES; ++w) {
            float4 x = *reinterpret_cast<const float4 *>(p + w * wstride);
            S.x += x.x; S.y += x.y; S.z += x.z; S.w += x.w;
        }
        store_dev128(out, idx * 16, S);
    }
}

// K split over workgroups, after the workgroup's last group: count this split in its group's
// counter; the workgroup that arrives last (the counter goes back to zero for the next launch)
// fetches all splits' partial tiles, chunk by chunk, into the slot buffer in split order and
// runs the epilogue on them.  The result does not depend on who arrives last; nothing waits.
__device__ __forceinline__ void split_finish(const PassArgs &a, int kind, int layer, const GemmPlan &pl, const StageLds &ly,
                                             const GemmEpi &ep, const Misc &mi, char *lds, int nt0, int n_local)
{
    const int tid = opaque(threadIdx.x);
    const int rows = a.rows, ks = 1 << pl.ksl;
    wait_vmem();      // this workgroup's partial tiles are visible device-wide ...
    __syncthreads();  // ... for every wave, before it is counted
    if (tid == 0) {
        int *cnt = a.sc.part_count + (blockIdx.x >> pl.ksl);
        const int before = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *mi.lastf = before == ks - 1 ? 1 : 0;
        if (*mi.lastf) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!*mi.lastf) return;
    float *slots = reinterpret_cast<float *>(lds);
    const size_t wstride = (size_t)ly.chunk * rows * 16;
    const WRes part = buffer_resource(a.sc.part);
    for (int c0 = 0; c0 < n_local; c0 += ly.chunk) {
        const int gn = min(ly.chunk, n_local - c0);
        const int per = gn * rows * 4;          // 16-byte items of one split's chunk
        for (int idx = tid; idx < ks * per; idx += WG_THREADS) {
            const int s = div_small(idx, per), rem = idx - s * per;
            // (byte offsets stay far below 2^31: the buffer holds splits x n-tiles x rows x 64 bytes)
            *reinterpret_cast<float4 *>(slots + s * wstride + (size_t)rem * 4) =
                load_dev128(part, (int)((((size_t)s * pl.NT + nt0 + c0) * rows * 16 + (size_t)rem * 4) * sizeof(float)));
        }
        lds_barrier();
        gemm_epilogue(a, kind, layer, ly, nt0 + c0, gn, rows, ep, mi, lds, ks);
        lds_barrier();
    }
}

// The streaming waves of a one-row-tile launch request the first EARLY_TILES tiles of their
// sequence as soon as the launch's arguments are there, before the plan arithmetic and the jump
// into the group's code (2 to 3 us on a cold instruction cache); the stage's first group takes
// them over.  The input copy is NOT moved forward with them: a compute unit holds about 64
// memory instructions in flight, whatever is requested first takes those slots, and the launch
// is shortest when the HBM requests go first and the copy follows once they are back
// (measured on the headline workload, ms per pass: neither early 3.38; tiles early 3.28; both
// early 3.37; copy early 3.47; tiles early and the copy right behind them 3.39; copy first,
// tiles behind it 3.45).
constexpr int EARLY_TILES = 8;
struct EarlyLoads {
    uint4 tile[EARLY_TILES];
};

template <int MT>
__device__ __forceinline__ void gemm_early(const GemmPlan &pl, const uint4 *__restrict__ W, EarlyLoads &early)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
    for (int i = 0; i < EARLY_TILES; ++i) early.tile[i] = make_uint4(0u, 0u, 0u, 0u);
    if constexpr (MT > 1) return;   // the accumulators of more row tiles need the registers
    int nt0, n_local;
    wg_units(pl, blockIdx.x, nt0, n_local);
    if (n_local <= 0 || wave >= SWAVES) return;
    const int nl = min(GROUP_TILES, n_local);
    const int last = max(wave_ksteps(pl.KTs, wave) * nl - 1, 0);
    const WRes wres = weight_resource(W);
    const int wstep = pl.nwg * SWAVES * 1024;
    const int woff = ((int)blockIdx.x * SWAVES + wave) * 1024;
#pragma unroll
    for (int i = 0; i < EARLY_TILES; ++i) early.tile[i] = load_tile16(wres, lane * 16, woff + min(i, last) * wstep);
}

// k-steps whose tiles a streaming wave keeps in flight, by n-tiles of the group: about 8 to 14
// tiles (1 KB each), fewer where the accumulators of three row tiles need the registers.  More
// does not stream faster: 12 and 16 tiles per wave measured the same pass time as 8 (what a
// compute unit can have in flight is bounded by the hardware, about 64 KB).
template <int MT, int NL>
constexpr int ring_steps()
{
    constexpr int r = (8 + NL - 1) / NL;
    return (MT == 3 && NL >= 5) ? 1 : r;
}

// One group of NL n-tiles (this workgroup's n-tiles nt_first .. nt_first + NL - 1) over all of K.
//
// Streaming wave w walks its k-steps s = 0 .. (k-tile w + SWAVES*s); per k-step it multiplies
// the NL weight tiles of the step with the step's input rows (two bf16 terms, MT row tiles)
// into NL x MT accumulators that stay in registers.  R k-steps of tiles are in flight: a step's
// registers are refilled with the step R further on as soon as the step has been used.  Every load
// is unconditional (the look-ahead is clamped to the group's last tile), nothing is pending
// when the loop is entered and no other memory operation of the wave goes through the vector
// path meanwhile: the compiler can then count the loads in flight and each use waits for
// exactly its own tile (otherwise it waits for all of them, which halves what a wave pulls).
//
// The input reaches LDS in blocks of ly.kbt k-tiles, copied by the helper waves through a ring
// of ly.nbuf buffers: later blocks are copied while block b is read; one barrier per block
// boundary, the same for all twelve waves.
//
// Afterwards the accumulators go through LDS, `ly.chunk` n-tiles at a time, for the
// cross-wave sum and the stage's epilogue (all waves).
template <int MT, int NL>
__device__ __forceinline__ void gemm_group(const PassArgs &a, int kind, int layer, const GemmPlan &pl, const StageLds &ly,
                                           const uint4 *__restrict__ W, const GemmIn &in, const GemmEpi &ep, const Misc &mi,
                                           char *lds, int nt_first, int seq0, bool first_group, const EarlyLoads &early)
{
    constexpr int R = ring_steps<MT, NL>();
    const ModelDev &md = a.mdv;
    const int tid = opaque(threadIdx.x), lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rows = a.rows;
    const int S_max = wave_ksteps(pl.KTs, 0);     // k-steps of the busiest wave: everybody runs the loop this far
    const int spb = ly.kbt / SWAVES;              // k-steps per input block
    f32x4_t acc[NL][MT];                          // streaming waves only

    if (wave < SWAVES) {
        // ---------------- streaming wave
#pragma unroll
        for (int nt = 0; nt < NL; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        const int S_w = wave_ksteps(pl.KTs, wave);
        const WRes wres = weight_resource(W);
        const int lane_off = lane * 16;
        const int wstep = pl.nwg * SWAVES * 1024;  // bytes from one tile of the wave's sequence to the next
        const int woff = ((seq0 * pl.nwg + (int)blockIdx.x) * SWAVES + wave) * 1024;  // the group's first tile
        const int last = max(S_w * NL - 1, 0);     // the group's last tile of this wave (look-ahead is clamped to it)
        uint4 buf[R][NL];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int nt = 0; nt < NL; ++nt) {
                const int i = r * NL + nt;
                if (MT == 1 && i < EARLY_TILES) {   // the stage's first group: requested at the start of the launch
                    buf[r][nt] = early.tile[i < EARLY_TILES ? i : 0];
                    if (!first_group) buf[r][nt] = load_tile16(wres, lane_off, woff + min(i, last) * wstep);
                } else {
                    buf[r][nt] = load_tile16(wres, lane_off, woff + min(i, last) * wstep);
                }
            }
        int brow[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) brow[mt] = min(mt * 16 + (lane & 15), rows - 1) * 64 + (lane >> 4) * 16;  // bytes inside a k-tile's hi rows
        const int tile_bytes = rows * 128;         // one k-tile of the input: both terms, all rows
        int blk_end = spb;                         // first k-step of the next input block
        int blk = 0, blk_buf = 0;                  // the block being read and its buffer of the ring
        int xoff = wave * tile_bytes;              // LDS byte offset of this wave's k-tile of step s, relative to s * SWAVES * tile_bytes
        wait_vmem();                               // nothing pending at loop entry (see above)
        lds_barrier();                             // input block 0 is in LDS
        for (int s0 = 0; s0 < S_max; s0 += R) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int s = s0 + r;
                if (s == blk_end && s < S_max) {   // next input block: the helpers have copied it into the next buffer of the ring
                    lds_barrier();
                    ++blk;
                    blk_buf = blk_buf + 1 == ly.nbuf ? 0 : blk_buf + 1;
                    xoff = wave * tile_bytes + blk_buf * ly.xbuf_bytes - blk * spb * SWAVES * tile_bytes;
                    blk_end += spb;
                }
                // A wave whose k-steps have run out keeps loading (its last tile again) and multiplies
                // with zeros: the stream loop then has no load under a condition.
                const bool live = s < S_w;
                const char *xs = lds + xoff + s * (SWAVES * tile_bytes);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {  // row tile by row tile: one pair of input operands live at a time
                    uint4 xh = make_uint4(0u, 0u, 0u, 0u), xl = xh;
                    if (live) {
                        xh = *reinterpret_cast<const uint4 *>(xs + brow[mt]);
                        xl = *reinterpret_cast<const uint4 *>(xs + brow[mt] + rows * 64);
                    }
                    const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, xh), bl = __builtin_bit_cast(bf16x8_t, xl);
#pragma unroll
                    for (int nt = 0; nt < NL; ++nt)  // the two terms of a tile in separate sweeps: no MFMA waits for the one before it
                        acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, buf[r][nt]), bh, acc[nt][mt], 0, 0, 0);
#pragma unroll
                    for (int nt = 0; nt < NL; ++nt) {
                        acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, buf[r][nt]), bl, acc[nt][mt], 0, 0, 0);
                        // the tile's registers are free after its last use: refill them with the step R further on
                        if (mt == MT - 1) buf[r][nt] = load_tile16(wres, lane_off, woff + min((s + R) * NL + nt, last) * wstep);
                    }
                }
            }
        }
    } else {
        // ---------------- helper wave: input blocks, row factors, per-row cache addresses
        const int hwave = wave - SWAVES;
        // Input blocks through a ring of ly.nbuf buffers: nbuf - 1 blocks are requested ahead of the
        // one being read, so that the copy of a block has the time of a whole block (or two) to arrive.
        // Block b is announced (barrier) once its own loads have landed, i.e. when only the loads of
        // the blocks requested after it are still pending.
        int issued = 0, cnt[3] = {0, 0, 0};        // cnt[j % 3]: load instructions of block j (nbuf <= 3)
        int next_buf = 0;                          // buffer of the ring the next requested block goes to (blocks are requested in order)
        auto request = [&](int j) __attribute__((always_inline)) {
            const int kt0 = j * ly.kbt;
            cnt[j % 3] = stage_block(in.x, rows, kt0, min(ly.kbt, pl.KTs - kt0), lds + next_buf * ly.xbuf_bytes, hwave, lane);
            next_buf = next_buf + 1 == ly.nbuf ? 0 : next_buf + 1;
        };
        for (; issued < max(ly.nbuf - 1, 1) && issued < ly.nkb; ++issued) request(issued);
        for (int b = 0; b < ly.nkb; ++b) {
            int after = 0;
            for (int j = b + 1; j < issued; ++j) after += cnt[j % 3];
            wait_vmem_pending(after);
            lds_barrier();                         // block b ready; block b-1 no longer read: its buffer takes the next request
            if (issued < ly.nkb) {
                request(issued);
                ++issued;
            }
        }
        // what only the epilogue needs, once the input is on its way: row factors, cache addresses
        // (ahead of the input copy they delayed the first MFMA of every launch by about 2 us)
        if (first_group) {
            if (in.ss) load_rstd(in.ss, a.nwg, md.rows_max, rows, pl.K, md.eps, mi.rstd, hwave, lane);
            const int ht = tid - SWAVES * 64;
            if (kind == G_QKV && ht < rows) {
                const int m = ht;
                const int pos = row_pos(a, m);
                const int ses = a.mode == 1 ? 0 : div_small(m, a.M);
                const int cbase = EE_SESS(a, ses, contig_base);
                const int page = cbase >= 0 ? cbase + pos / KV_PAGE : as_global(EE_SESS(a, ses, page_table))[pos / KV_PAGE];
                mi.pos[m] = pos;
                mi.kvoff[m] = (((long long)layer * EE_SESS(a, ses, n_pages) + page) * md.H) * KV_PAGE * 2 * md.hd;  // record of head 0
            }
            wait_vmem();
        }
    }
    // ---- cross-wave sum and epilogue, ly.chunk n-tiles at a time (the input buffers are free now)
    lds_barrier();                                 // every streaming wave is done with the input
    float *slots = reinterpret_cast<float *>(lds);
    for (int c0 = 0; c0 < NL; c0 += ly.chunk) {
        const int gn = min(ly.chunk, NL - c0);
        if (wave < SWAVES) {
            // D layout: lane holds rows (lane>>4)*4 .. +3 of N, column (lane&15) of M
#pragma unroll
            for (int nt = 0; nt < NL; ++nt)
                if (nt >= c0 && nt < c0 + gn) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const int m = mt * 16 + (lane & 15);
                        if (m < rows)
                            *reinterpret_cast<float4 *>(slots + (((size_t)wave * ly.chunk + (nt - c0)) * rows + m) * 16 + (lane >> 4) * 4) =
                                make_float4(acc[nt][mt][0], acc[nt][mt][1], acc[nt][mt][2], acc[nt][mt][3]);
                    }
                }
        }
        lds_barrier();
        if (MT > 1 && pl.ksl)   // (K is split only for launches of more than one row tile)
            partial_store(a, pl, ly, nt_first + c0, gn, rows, lds);
        else
            gemm_epilogue(a, kind, layer, ly, nt_first + c0, gn, rows, ep, mi, lds, SWAVES);
        lds_barrier();
    }
}

// One GEMM stage of this workgroup: its n-tiles in groups of up to GROUP_TILES.
template <int MT>
__device__ __forceinline__ void gemm_stage_t(const PassArgs &a, int kind, int layer, const GemmPlan &pl, const StageLds &ly,
                             const uint4 *__restrict__ W, const GemmIn &in_all, const GemmEpi &ep, char *lds, const EarlyLoads &early)
{
    const ModelDev &md = a.mdv;
    const int tid = opaque(threadIdx.x);
    const int rows = a.rows;
    const Misc mi = misc_views(ly, lds);
    int nt0, n_local;
    wg_units(pl, blockIdx.x, nt0, n_local);

    if (tid < rows) {
        mi.bestv[tid] = -INFINITY;
        mi.besti[tid] = 0x7FFFFFFF;
        mi.sume[tid] = 0.f;
        mi.rowss[tid] = 0.f;
    }
    if (n_local > 0) {
        const int S0 = wave_ksteps(pl.KTs, 0);
        // K split over workgroups: this workgroup's slice of the input (k-tile-major: a contiguous range)
        const GemmIn in = {MT > 1 ? in_all.x + (size_t)(blockIdx.x & ((1 << pl.ksl) - 1)) * pl.KTs * (2 * rows * 32) : in_all.x, in_all.ss};
        int seq = 0;  // tiles of a wave's sequence before the group (waves with fewer k-steps leave their slots unused)
        for (int g0 = 0; g0 < n_local; g0 += GROUP_TILES) {
            const int nl = min(GROUP_TILES, n_local - g0);
            const bool first = g0 == 0;
#define EE_GROUP(NLV) \
    case NLV: gemm_group<MT, NLV>(a, kind, layer, pl, ly, W, in, ep, mi, lds, nt0 + g0, seq, first, early); break;
            switch (nl) {
                EE_GROUP(1) EE_GROUP(2) EE_GROUP(3) EE_GROUP(4) EE_GROUP(5) EE_GROUP(6) EE_GROUP(7) EE_GROUP(8)
            }
#undef EE_GROUP
            seq += S0 * nl;
        }
        if (MT > 1 && pl.ksl) split_finish(a, kind, layer, pl, ly, ep, mi, lds, nt0, n_local);
    }
    // what the workgroup hands to the following launch
    auto hand_over = [&](int slot, bool mine) __attribute__((always_inline)) {
        const float ss = mine ? mi.rowss[tid] : 0.f;
        if (ep.ss_out) as_global_mut(ep.ss_out)[(size_t)slot * md.rows_max + tid] = ss;
        if (ep.ss_head) as_global_mut(ep.ss_head)[(size_t)slot * md.rows_max + a.head_row0 + tid] = ss;
        if (kind == G_HEAD) {  // device-scope stores: the accept step may run in another workgroup of this launch
            store_dev64(a.sc.cand + (size_t)slot * md.rows_max + tid,
                        make_uint2(__float_as_uint(mine ? mi.bestv[tid] : -INFINITY), (unsigned)(mine ? mi.besti[tid] : 0x7FFFFFFF)));
            store_dev32(a.sc.cand_sum + (size_t)slot * md.rows_max + tid, mine ? mi.sume[tid] : 0.f);
        }
    };
    if (tid < rows) {
        if (MT > 1 && pl.ksl && n_local > 0) {
            // K split: the group's result was worked out by whichever of its workgroups arrived last; it
            // fills the slots of the whole group, the result in the first, so that what the following
            // launch adds up (in slot order) does not depend on who that was
            if (*mi.lastf) {
                const int ks = 1 << pl.ksl, first = (int)blockIdx.x & ~(ks - 1);
                for (int j = 0; j < ks; ++j) hand_over(first + j, j == 0);
            }
        } else {
            hand_over((int)blockIdx.x, true);
        }
    }
}

// ------------------------------------------------------------------ embedding

// h = embedding of each row's token (or the supplied embedding row); workgroup g owns the
// columns [g*cw, (g+1)*cw) and also emits the first layer's GEMM input and its share of h^2
__device__ __forceinline__ void embed_stage(const PassArgs &a, char *lds)
{
    const ModelDev &md = a.mdv;
    const int d = md.d, rows = a.rows, tid = threadIdx.x;
    const int cw = (div_small(d + a.nwg - 1, a.nwg) + 3) & ~3;  // columns per workgroup, multiple of 4
    const int n0 = blockIdx.x * cw;
    const int nq = max(0, min(cw, d - n0)) >> 2;          // quads of columns here
    float *sq = reinterpret_cast<float *>(lds);           // [rows][cw/4]
    const float *gain = md.g_attn + (size_t)a.layer_begin * d;
    for (int it = tid; it < rows * nq; it += WG_THREADS) {
        int m = div_small(it, nq), c = n0 + (it - m * nq) * 4;
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
        as_global_mut(a.sc.ss_a)[(size_t)blockIdx.x * md.rows_max + tid] = t;
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
__device__ __forceinline__ void att_stage(const PassArgs &a, int layer, char *lds)
{
    constexpr int KT = HD / 32;  // 32-value steps of a score
    constexpr int NT = HD / 16;  // 16-column tiles of the output
    constexpr int REC = HD + 2;
    const int H = a.H, d = a.d, M = a.M;  // copies in the launch arguments: no load before the first address
    const int n_chunks = (M + ATT_ROWS - 1) / ATT_ROWS;
    const int n_splits = a.att_splits;
    const int n_items = a.n_sess * H * n_chunks * n_splits;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lm = lane & 15, quad = lane >> 4;
    float *wbuf = reinterpret_cast<float *>(lds);  // [WAVES][ATT_ROWS][REC]
    int *lastf = reinterpret_cast<int *>(wbuf + (size_t)WAVES * ATT_ROWS * REC);
    const size_t rec_page = (size_t)KV_PAGE * 2 * HD;  // elements of one (page, head) record
    for (int item = blockIdx.x; item < n_items; item += a.nwg) {
        int unit = div_small(item, n_splits), sp = item - unit * n_splits;
        int s = div_small(unit, H * n_chunks), rem = unit - s * (H * n_chunks);
        int hh = div_small(rem, n_chunks), ch = rem - hh * n_chunks;
        int r0 = ch * ATT_ROWS, nr = min(ATT_ROWS, M - r0);
        // session 0's descriptor also travels by value in the launch arguments: no dependent load
        const int *page_table = EE_SESS(a, s, page_table);
        const uint16_t *kpool = EE_SESS(a, s, kpool);
        const uint16_t *vpool = EE_SESS(a, s, vpool);
        const int n_pages = EE_SESS(a, s, n_pages);
        const int P = a.mode == 1 ? a.pf_pos0 : EE_SESS(a, s, kv_len);  // position of the first row
        const int n_pos = P + r0 + nr;  // positions visible to the chunk's last row
        const int n_pg = (n_pos + KV_PAGE - 1) / KV_PAGE;
        const int pg_lo = div_small(n_pg * sp, n_splits), pg_hi = div_small(n_pg * (sp + 1), n_splits);
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
            wait_vmem();      // this item's partials are visible device-wide ...
            __syncthreads();  // ... for every wave, before it is counted
            if (tid == 0) {
                int before = __hip_atomic_fetch_add(a.sc.att_count + unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *lastf = before == n_splits - 1 ? 1 : 0;
            }
            __syncthreads();
            if (*lastf) {
                // (the split count goes through an opaque copy here: otherwise everything below that
                // depends only on it -- sixteen clamped offsets, sixteen conditions -- is worked out
                // at the start of the kernel, by every workgroup, before its first load)
                const int n_splits = opaque(a.att_splits);
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
__device__ __forceinline__ void accept_stage(const PassArgs &a, char *lds)
{
    const ModelDev &md = a.mdv;
    const int rows = a.rows, M = a.M;  // rows of the head launch: head after head, session after session, M rows each
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int *tok = reinterpret_cast<int *>(lds);
    float *conf = reinterpret_cast<float *>(lds) + EE_MAX_ROWS;
    for (int m = wave; m < rows; m += WAVES) {
        // all of the row's candidates and partial sums are requested before the first is used
        constexpr int PER = 4;                     // workgroups per lane: the launch has at most 256
        int2 c[PER];
        float sg[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int g = lane + 64 * j;
            c[j] = make_int2(__float_as_int(-INFINITY), 0x7FFFFFFF);
            sg[j] = 0.f;
            if (g < a.nwg) {
                c[j] = load_cand(a.sc.cand + (size_t)g * md.rows_max + m);
                sg[j] = load_dev32(a.sc.cand_sum + (size_t)g * md.rows_max + m);
            }
        }
        float bv = -INFINITY;
        int bi = 0x7FFFFFFF;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const float v = __int_as_float(c[j].x);
            if (cand_better(v, c[j].y, bv, bi)) {
                bv = v;
                bi = c[j].y;
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
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (sg[j] > 0.f) se += sg[j] * __expf(__int_as_float(c[j].x) - bv);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) se += __shfl_xor(se, off, 64);
        if (lane == 0) {
            tok[m] = bi;
            conf[m] = 1.0f / se;
        }
    }
    __syncthreads();
    // one thread per (head of this launch, session)
    if ((int)threadIdx.x < a.n_heads * a.n_sess) {
        const int hj = div_small(threadIdx.x, a.n_sess), s = threadIdx.x - hj * a.n_sess, head = a.head_idx + hj;
        const SessDev &sd = a.sess[s];
        ee_verify_result *res = sd.result;
        const int *t = tok + (hj * a.n_sess + s) * M;
        const float *cf = conf + (hj * a.n_sess + s) * M;
        if (a.head_kind == HEAD_PREFILL) {
            int last = t[M - 1];
            res->next_token = last;
            res->device_status = 0;
            sd.state[1] = last;
        } else {
            const int gamma = M - 1;
            int delta = 0;
            if (a.sm.on) {
                // probabilistic verification: the rows' decisions were taken by the sampling launch;
                // the tokens published are the ones each row emits if the round ends there
                int *ts = tok + (hj * a.n_sess + s) * M;
                unsigned kept = 0;
                for (int i = 0; i < M; ++i) {
                    const int r = (hj * a.n_sess + s) * M + i;   // the row of the head launch
                    ts[i] = __hip_atomic_load(a.sm.tok + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (i < gamma && __hip_atomic_load(a.sm.kept + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) kept |= 1u << i;
                }
                delta = __builtin_ctz(~kept);   // drafts kept before the first one that is not (bit gamma is never set)
            } else {
                int dr[EE_MAX_M];
#pragma unroll
                for (int i = 0; i < EE_MAX_M - 1; ++i) dr[i] = i < gamma ? sd.drafts[i] : -1;
#pragma unroll
                for (int i = 0; i < EE_MAX_M - 1; ++i)
                    if (delta == i && i < gamma && dr[i] == t[i]) delta = i + 1;
            }
            if (a.head_kind == HEAD_EXIT) {
                for (int i = 0; i < M; ++i) {
                    res->exit_tokens[head][i] = t[i];
                    res->exit_conf[head][i] = cf[i];
                }
                res->exit_accept_len[head] = delta;
            } else {
                for (int i = 0; i < M; ++i) {
                    res->final_tokens[i] = t[i];
                    res->final_conf[i] = cf[i];
                }
                res->accept_len = delta;
                res->next_token = t[delta];
                res->device_status = 0;
                if (a.commit) {
                    sd.state[0] = sd.state[0] + delta + 1;
                    sd.state[1] = t[delta];
                }
            }
        }
        __threadfence_system();
    }
}

// ------------------------------------------------------------------ probabilistic verification

// Weights of the cumulative sums are 40-bit fixed point (integers): their sums do not depend on
// the order of addition, so every thread's share [exclusive sum, + own sum) of the cumulative
// distribution tiles it exactly and the search below always ends inside the owner's tokens.
// A weight is at most 1 (largest exp term, or a probability) and a row has at most 2^15 tokens.
typedef unsigned long long u64;
constexpr int SAMPLE_LDS_BYTES = 4096;             // the waves' sums and flags; the accept step's rows
constexpr float SAMPLE_UNIT = 1099511627776.0f;  // 2^40

__device__ __forceinline__ u64 fixed_weight(float w) { return (u64)(w * SAMPLE_UNIT); }

// e_k = exp((z_k - zmax) / T): un-normalised probability of token k under the target distribution
__device__ __forceinline__ float target_term(float z, float zmax, float inv_T) { return expf((z - zmax) * inv_T); }

// positive part of q_k - p_k (one fused multiply-add, so that every place that forms it gets the same bits)
__device__ __forceinline__ float residual_term(float e, float inv_Z, float p) { return fmaxf(__fmaf_rn(e, inv_Z, -p), 0.f); }

// sum of one 64-bit value per lane over the wave (every lane gets it)
__device__ __forceinline__ u64 wave_sum(u64 x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

constexpr int SAMPLE_CH = 22;   // blocks of 64 tokens a wave requests in one go (all loads in flight together)

// values first + 64 j + lane, j < SAMPLE_CH, of a row; `fill` past the end t1
__device__ __forceinline__ void load_chunk(const EE_GLOBAL float *row, int first, int t1, int lane, float fill, float (&out)[SAMPLE_CH])
{
#pragma unroll
    for (int j = 0; j < SAMPLE_CH; ++j) {
        const int k = first + 64 * j + lane;
        out[j] = k < t1 ? row[k] : fill;
    }
}

// One row of one head under probabilistic verification (Eq. 2 / Eq. 5 of the paper with the
// draft model's distributions; the keep / replace rule of the speculative sampling scheme the
// paper builds on).  q = softmax(z / T) of the row's logits.  Row i < gamma: its draft x is kept
// iff u_i * p_i(x) < q(x), and if the round ends here the row emits a token drawn from the
// positive part of q - p_i; row gamma emits a token drawn from q.  Drawing = inversion of the
// cumulative sum in token order with the row's number v_i: the first token whose cumulative
// weight exceeds v_i * (sum of the weights).
//
// Wave w owns the tokens [w * S, (w + 1) * S) and walks them in chunks of SAMPLE_CH blocks of
// 64 (lane l: token first + 64 j + l, coalesced; a chunk's loads are all requested before the
// first is used: a pass over the row costs one memory latency per chunk, not one per token).
// The sums are integers, so the cumulative sum up to a token is the earlier waves' totals + this
// wave's earlier blocks + a scan inside the block, whatever the order they were added in.
__device__ __forceinline__ void sample_stage(const PassArgs &a, int r, char *lds)
{
    static_assert(WAVES * 8 * 2 + WAVES * 4 + 16 <= SAMPLE_LDS_BYTES && EE_MAX_ROWS * 8 <= SAMPLE_LDS_BYTES, "LDS of the sampling launch");
    const int V = a.mdv.V, M = a.M, gamma = M - 1;
    const int per_head = a.n_sess * M;                          // the launch's rows: head after head, session after session
    const int hj = div_small(r, per_head), rr = r - hj * per_head;
    const int ses = div_small(rr, M), i = rr - ses * M;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    u64 *wtot = reinterpret_cast<u64 *>(lds);                   // [WAVES] the waves' totals (target terms)
    u64 *rtot = wtot + WAVES;                                   // [WAVES] the same for the residual weights
    float *wmax = reinterpret_cast<float *>(rtot + WAVES);      // [WAVES]
    int *found = reinterpret_cast<int *>(wmax + WAVES);
    const EE_GLOBAL float *z = as_global(a.sc.logits) + ((size_t)(a.head_idx + hj) * a.mdv.rows_max + rr) * V;
    const EE_GLOBAL float *p = as_global(a.sm.probs) + ((size_t)ses * gamma + min(i, gamma - 1)) * V;
    const EE_GLOBAL float *uv = as_global(a.sm.uv) + (size_t)ses * (2 * gamma + 2);   // the session's u, v and 1 / temperature
    const float inv_T = uv[2 * gamma + 1];
    const int S = ((V + WAVES - 1) / WAVES + 63) & ~63;         // tokens per wave, whole blocks of 64
    const int t0 = min(V, wave * S), t1 = min(V, t0 + S);
    constexpr int CHUNK = SAMPLE_CH * 64;
    float zc[SAMPLE_CH], pc[SAMPLE_CH];

    // largest logit
    float mx = -INFINITY;
    for (int c0 = t0; c0 < t1; c0 += CHUNK) {
        load_chunk(z, c0, t1, lane, -INFINITY, zc);
#pragma unroll
        for (int j = 0; j < SAMPLE_CH; ++j) mx = fmaxf(mx, zc[j]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (lane == 0) wmax[wave] = mx;
    if (tid == 0) *found = 0;
    __syncthreads();
    float zmax = wmax[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) zmax = fmaxf(zmax, wmax[w]);

    // Z = sum_k e_k  (a logit of -inf past the row's end contributes exp(-inf) = 0)
    u64 part = 0;
    for (int c0 = t0; c0 < t1; c0 += CHUNK) {
        load_chunk(z, c0, t1, lane, -INFINITY, zc);
#pragma unroll
        for (int j = 0; j < SAMPLE_CH; ++j) part += fixed_weight(target_term(zc[j], zmax, inv_T));
    }
    part = wave_sum(part);
    if (lane == 0) wtot[wave] = part;
    __syncthreads();
    u64 Zi = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) Zi += wtot[w];
    const float inv_Z = 1.0f / (float)((double)Zi * (1.0 / (double)SAMPLE_UNIT));

    const u64 *tot = wtot;
    u64 w_total = Zi;
    bool residual = false;
    int kept = 0;
    if (i < gamma) {
        const int x = as_global(EE_SESS(a, ses, drafts))[i];
        const float qx = target_term(z[x], zmax, inv_T) * inv_Z;
        kept = uv[i] * p[x] < qx ? 1 : 0;
        u64 rp = 0;
        for (int c0 = t0; c0 < t1; c0 += CHUNK) {
            load_chunk(z, c0, t1, lane, -INFINITY, zc);
            load_chunk(p, c0, t1, lane, 0.f, pc);
#pragma unroll
            for (int j = 0; j < SAMPLE_CH; ++j) rp += fixed_weight(residual_term(target_term(zc[j], zmax, inv_T), inv_Z, pc[j]));
        }
        rp = wave_sum(rp);
        if (lane == 0) rtot[wave] = rp;
        __syncthreads();
        u64 W = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) W += rtot[w];
        if (W > 0) {  // otherwise q = p: the draft is always kept and the row never emits; it then draws from q
            residual = true;
            tot = rtot;
            w_total = W;
        }
    }
    // the first token whose cumulative weight exceeds the target; v < 1, so target < w_total
    const double vd = (double)uv[gamma + i];
    u64 target = (u64)(vd * (double)w_total);
    if (target >= w_total) target = w_total - 1;
    u64 before = 0;                                              // cumulative weight of the waves before this one
    for (int w = 0; w < wave; ++w) before += tot[w];
    if (before <= target && target < before + tot[wave]) {      // exactly one wave
        u64 run = before;
        bool done = false;
        for (int c0 = t0; c0 < t1 && !done; c0 += CHUNK) {
            load_chunk(z, c0, t1, lane, -INFINITY, zc);
            if (residual) load_chunk(p, c0, t1, lane, 0.f, pc);
            // the blocks' sums first, all of them (independent reductions overlap), then the search
            u64 wk[SAMPLE_CH], blk[SAMPLE_CH];
#pragma unroll
            for (int j = 0; j < SAMPLE_CH; ++j) {
                const float e = target_term(zc[j], zmax, inv_T);
                wk[j] = fixed_weight(residual ? residual_term(e, inv_Z, pc[j]) : e);
            }
#pragma unroll
            for (int j = 0; j < SAMPLE_CH; ++j) {
                const u64 t = wave_sum(wk[j]);
                blk[j] = ((u64)(unsigned)__builtin_amdgcn_readfirstlane((int)(t >> 32)) << 32) | (unsigned)__builtin_amdgcn_readfirstlane((int)t);
            }
            int jh = -1;
            u64 mine = 0;
#pragma unroll
            for (int j = 0; j < SAMPLE_CH; ++j)
                if (jh < 0) {
                    if (run + blk[j] > target) {
                        jh = j;
                        mine = wk[j];
                    } else {
                        run += blk[j];
                    }
                }
            if (jh >= 0) {                                       // the token is in block jh: scan it
                u64 incl = mine;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const u64 o = __shfl_up(incl, off, 64);
                    if (lane >= off) incl += o;
                }
                const unsigned long long hit = __ballot(run + incl > target);
                if (lane == 0) *found = c0 + 64 * jh + __builtin_ctzll(hit);
                done = true;
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        __hip_atomic_store(a.sm.tok + r, *found, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.sm.kept + r, kept, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ------------------------------------------------------------------ kernels of the pass
//
// Stage list of a segment: [EMBED] { QKV ATT O GU DN } x layers [HEAD]; one launch per stage.
// The accept step runs inside the head's launch, in the workgroup that finishes last.

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
    if (a.head_kind != HEAD_NONE) {  // [AD AU] [HEAD]
        const int n_ad = a.adapter ? 2 : 0;
        if (idx < n_ad) {
            sd.type = ST_GEMM;
            sd.kind = G_AD + idx;
        } else if (idx == n_ad && a.head_stage) {
            sd.type = ST_GEMM;
            sd.kind = G_HEAD;
        }
    }
    return sd;
}

__device__ __forceinline__ GemmIn gemm_input(const PassArgs &a, int kind)
{
    switch (kind) {
    case G_QKV: return GemmIn{a.sc.xn, a.sc.ss_a};
    case G_O: return GemmIn{a.sc.attn, nullptr};
    case G_GU: return GemmIn{a.sc.xn, a.sc.ss_f};
    case G_DN: return GemmIn{a.sc.u, nullptr};
    case G_AD: return GemmIn{a.sc.xa, nullptr};
    case G_AU: return GemmIn{a.sc.t, nullptr};
    default: return GemmIn{a.sc.xh, a.sc.ss_h};
    }
}

__device__ __forceinline__ GemmEpi gemm_epi(const PassArgs &a, int kind, int layer)
{
    const ModelDev &md = a.mdv;
    GemmEpi ep = {nullptr, nullptr, nullptr, nullptr, nullptr, 0};
    if (kind == G_O) {
        ep.gain_xn = md.g_ffn + (size_t)layer * md.d;
        ep.ss_out = a.sc.ss_f;
    } else if (kind == G_DN) {
        if (layer + 1 < md.L) ep.gain_xn = md.g_attn + (size_t)(layer + 1) * md.d;
        if (layer + 1 == a.layer_end && a.head_kind != HEAD_NONE) {
            if (a.adapter) {
                ep.xa_out = 1;                 // the exit's adapters come first
            } else {
                ep.gain_xh = a.head_gain;      // the LM head's input rows and their sums of squares
                ep.ss_head = a.sc.ss_h;
            }
        }
        ep.ss_out = a.sc.ss_a;
    } else if (kind == G_AD) {
        ep.bias = a.ad_bdown;
    } else if (kind == G_AU) {
        ep.bias = a.ad_bup;
        ep.gain_xh = a.head_gain;
        ep.ss_head = a.sc.ss_h;
    }
    return ep;
}

// The GEMM stage a.stage of the stage list.  MT = 16-row tiles of the pass (rows <= 16 * MT).
template <int MT>
__global__ void __launch_bounds__(WG_THREADS) ee_gemm_kernel(PassArgs a_by_value)
{
    extern __shared__ __align__(16) char lds[];
    const PassArgs &a = warmed_arguments();
    EarlyLoads early;
    gemm_early<MT>(a.plan0, a.W0, early);
    const StageDesc st = stage_decode(a, a.stage);
    gemm_stage_t<MT>(a, st.kind, st.layer, a.plan0, a.lay, a.W0, gemm_input(a, st.kind), gemm_epi(a, st.kind, st.layer), lds, early);
    if (a.fuse_accept) {
        // A head stage: the workgroup whose candidates arrive last also runs the accept step
        // (one launch less per head); the counter is left at zero.
        int *lastf = misc_views(a.lay, lds).lastf;
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
}

// Probabilistic verification: one workgroup per row of the head launch before it (whose logits
// it reads); the workgroup that finishes last applies the accept rule and publishes, as the
// head launch's last workgroup does under exact-match verification.
__global__ void __launch_bounds__(WG_THREADS) ee_sample_kernel(PassArgs a_by_value)
{
    extern __shared__ __align__(16) char lds[];
    const PassArgs &a = warmed_arguments();
    sample_stage(a, blockIdx.x, lds);
    int *lastf = reinterpret_cast<int *>(lds + SAMPLE_LDS_BYTES - 16);   // behind sample_stage's and the accept step's arrays
    wait_vmem();
    __syncthreads();
    if (threadIdx.x == 0) {
        const int before = __hip_atomic_fetch_add(a.sm.count, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *lastf = before == (int)gridDim.x - 1 ? 1 : 0;
        if (*lastf) __hip_atomic_store(a.sm.count, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (*lastf) accept_stage(a, lds);
}

template <int HD>
__global__ void __launch_bounds__(WG_THREADS) ee_att_kernel(PassArgs a_by_value)
{
    extern __shared__ __align__(16) char lds[];
    const PassArgs &a = warmed_arguments();
    att_stage<HD>(a, stage_decode(a, a.stage).layer, lds);
}

// embedding
__global__ void __launch_bounds__(WG_THREADS) ee_misc_kernel(PassArgs a_by_value)
{
    extern __shared__ __align__(16) char lds[];
    const PassArgs &a = warmed_arguments();
    if (stage_decode(a, a.stage).type == ST_EMBED) embed_stage(a, lds);
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
// sub-wave `sub` of the block those of streaming wave w = sub, sub + nsub, ...
__global__ void tile_weights_kernel(const uint16_t *__restrict__ src, uint4 *__restrict__ dst, GemmPlan pl,
                                    int perm, int d, int hd, int F)
{
    const int g = blockIdx.x;
    int nt0, n_local;
    wg_units(pl, g, nt0, n_local);
    if (n_local == 0) return;
    const int lane = threadIdx.x & 63, sub = threadIdx.x >> 6, nsub = blockDim.x >> 6;
    const int S0 = wave_ksteps(pl.KTs, 0);
    const int kt_first = (g & ((1 << pl.ksl) - 1)) * pl.KTs;   // K split over workgroups: this workgroup's slice
    for (int w = sub; w < SWAVES; w += nsub) {
        const int S_w = wave_ksteps(pl.KTs, w);
        int seq = 0;
        for (int g0 = 0; g0 < n_local; g0 += GROUP_TILES) {
            const int nl = min(GROUP_TILES, n_local - g0);
            for (int s = 0; s < S_w; ++s)
                for (int nt = 0; nt < nl; ++nt) {
                    int n = (nt0 + g0 + nt) * 16 + (lane & 15);
                    int k0 = (kt_first + w + SWAVES * s) * 32 + (lane >> 4) * 8;
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
                    const size_t step = (size_t)seq + (size_t)s * nl + nt;
                    dst[((step * pl.nwg + g) * SWAVES + w) * 64 + lane] = o;
                }
            seq += S0 * nl;
        }
    }
}

// counts the x in [0, x_max] with div_small(x, d) != x / d, for every divisor of the list
__global__ void div_small_check_kernel(const int *__restrict__ divisors, int n_div, int x_max, unsigned long long *bad)
{
    unsigned long long mine = 0;
    for (int j = blockIdx.y; j < n_div; j += gridDim.y) {
        const int d = divisors[j];
        for (long long x = (long long)blockIdx.x * blockDim.x + threadIdx.x; x <= x_max; x += (long long)gridDim.x * blockDim.x)
            mine += div_small((int)x, d) != (int)x / d ? 1 : 0;
    }
    if (mine) atomicAdd(bad, mine);
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
