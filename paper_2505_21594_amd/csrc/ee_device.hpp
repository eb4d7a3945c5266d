// Structures shared by the host runtime and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ee.h"

namespace ee {

constexpr int SWAVES = 8;                // streaming waves: weight tiles -> MFMA
constexpr int HWAVES = 4;                // helper waves: stage the input blocks while the others stream
constexpr int WAVES = SWAVES + HWAVES;   // three per SIMD, 168 VGPRs each
constexpr int WG_THREADS = WAVES * 64;
constexpr int GROUP_TILES = 8;           // n-tiles whose accumulators a streaming wave keeps in registers at once
constexpr int KV_PAGE = 16;              // positions per KV page
constexpr int ATT_ROWS = 16;             // query rows of one attention item (one MFMA tile)
constexpr int ATT_TILES = 8;             // KV pages (score tiles) a wave keeps in registers per item
constexpr int ATT_MAX_SPLITS = 16;
constexpr int KSPLIT_LOG2 = 2;           // many-row launches: workgroups (1 << this) that share n-tiles and split K (at most SWAVES)

// Weight layout of one GEMM y = x . W^T, W[N][K] row-major in the model file.
//
// A tile is the A operand of one v_mfma_f32_16x16x32_bf16: 16 rows of N by 32
// columns of K, stored as 64 lanes x 16 bytes, lane l holding
// W[nt*16 + (l & 15)][kt*32 + (l >> 4)*8 .. +7]  (1 KB per tile).
//
// The N axis is cut into units of `tpu` n-tiles (1, or 2 for a gate/up pair);
// workgroup g owns a contiguous range of units (unit_range below) for the whole of K, so
// every output element is complete inside one workgroup.  Its n-tiles are taken in groups
// of up to GROUP_TILES; streaming wave w owns the k-tiles w, w + SWAVES, w + 2 SWAVES, ...
// ("k-steps" s = 0, 1, ...) and walks
//   for group : for k-step s : for n-tile of the group : tile(n-tile, k-tile w + SWAVES*s)
// keeping one accumulator per n-tile of the group in registers for the whole of K.  The order
// does not depend on the number of rows; how many k-tiles of the input sit in LDS at a time
// (StageLds) is chosen per launch.
// In memory the tiles are interleaved over the whole chip: the i-th tile of the
// sequence of wave w of workgroup g sits at tile slot (i*nwg + g)*SWAVES + w, so at any
// moment all waves together read one contiguous window (measured: up to 15 % more
// HBM bandwidth than one contiguous range per wave).  `steps` is the longest sequence.
struct GemmPlan {
    int N, K;        // logical shape (N counts rows after concatenation / interleaving)
    int NT, KT;      // tiles along N and K (K zero-padded to 32)
    int tpu;         // n-tiles per unit
    int U;           // units = NT / tpu
    int steps;       // tile slots per wave (longest wave sequence)
    int nwg;         // workgroups that take part in this stage kind: the fewest that keep the busiest one's
                     // share unchanged, so that all of them get (nearly) the same share; the rest idle.
                     // Half of the compute units already saturate HBM, uneven shares only lengthen the tail.
    // K split over workgroups (many-row launches): 1 << ksl consecutive workgroups share the same
    // n-tiles and take one slice of KTs k-tiles each (workgroup g: n-tiles of g >> ksl, slice
    // g & (splits - 1)); their partial tiles meet in memory and the one that arrives last adds them
    // up and runs the epilogue.  A workgroup then copies only its slice of the input into LDS and
    // has 1 << ksl times the n-tiles per input block.  ksl = 0, KTs = KT: no split.
    int ksl, KTs;
};

// LDS map of one GEMM launch, chosen on the host from the rows of the launch:
//   [input buffer 0][input buffer 1][input buffer 2] ... [misc]
// An input block holds kbt k-tiles of the input as [k-tile][term][row][32] bf16 (both bf16
// terms, all rows); with nkb > 1 blocks the helper waves fill the other buffers of a ring of
// nbuf (2, or 3 when many rows leave room for short blocks only) while the streaming waves read one.  After a group's last block the same space holds the waves'
// partial tiles for the cross-wave sum ([wave][n-tile of the chunk][row][16] floats, `chunk`
// n-tiles at a time) and, behind them at zbuf_off, one [row][chunk*16] float tile for the
// head's logits / the squares of the residual stream.
struct StageLds {
    int kbt;         // k-tiles per input block (a multiple of SWAVES)
    int nkb;         // input blocks along K
    int nbuf;        // input buffers (1 when the whole of K fits one)
    int xbuf_bytes;  // bytes of one input buffer
    int chunk;       // n-tiles reduced at a time
    int zbuf_off;
    int misc_off;
};

// Units [u0, u1) of workgroup g.  Workgroups are dealt to the chip's 8 XCDs round-robin (XCD =
// g % 8) and every XCD has its own path to memory, so the units are first split evenly over
// the XCDs and then over the XCD's workgroups: with U not a multiple of nwg, a plain split
// over g loads some XCDs up to 20 % more than others and the launch ends with them.
constexpr int NUM_XCD = 8;
// x / d for 0 <= x <= DIV_SMALL_MAX and d >= 1.  The GPU has no integer division: a 32-bit one is
// about 40 instructions in a dependent chain, a 64-bit one several hundred, and the kernels divide
// by run-time values on the way to their first load, at every block boundary of the stream and in
// every epilogue item.  One reciprocal (1 ulp) and one multiply give the exact quotient in this
// range: (x + 0.5) / d is at least 0.5 / d away from an integer and the error of the product is
// below (x + 0.5) / d * 1.8e-7, which is less than 0.5 / d for x < 2.7e6.
constexpr int DIV_SMALL_MAX = 2500000;
__host__ __device__ inline int div_small(int x, int d)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return (int)(((float)x + 0.5f) * __builtin_amdgcn_rcpf((float)d));
#else
    return x / d;
#endif
}

// (host: U * nwg <= DIV_SMALL_MAX is checked when the model is loaded)
__host__ __device__ inline void unit_range(int U, int nwg, int g, int &u0, int &u1)
{
    if (nwg % NUM_XCD != 0) {
        u0 = div_small(U * g, nwg);
        u1 = div_small(U * (g + 1), nwg);
        return;
    }
    const int x = g % NUM_XCD, j = g / NUM_XCD, per = nwg / NUM_XCD;
    const int x0 = U * x / NUM_XCD, x1 = U * (x + 1) / NUM_XCD;
    u0 = x0 + div_small((x1 - x0) * j, per);
    u1 = x0 + div_small((x1 - x0) * (j + 1), per);
}

enum RowPerm { PERM_NONE = 0, PERM_QKV = 1, PERM_GU = 2 };
enum GemmKind { G_QKV = 0, G_O = 1, G_GU = 2, G_DN = 3, G_HEAD = 4, G_AD = 5, G_AU = 6, G_KINDS = 7 };  // AD / AU: an exit head's adapter, down and up
enum StageType { ST_EMBED = 0, ST_GEMM = 1, ST_ATT = 2, ST_ACCEPT = 3, ST_NONE = 4 };

struct ModelDev {
    int L, d, H, hd, F, V;
    float eps, att_scale;
    int Kpad_d, Kpad_F;                  // K rounded up to 32
    int rows_max;
    int A, Kpad_A;                       // hidden units of an exit head's adapters (all bottlenecks together; 0: none), rounded up to 32
    const float *g_attn, *g_ffn;         // [L][d]
    const float *g_final;
    const uint16_t *emb;                 // [V][d] bf16, row-major
};

struct SessDev {
    int *state;                          // [0] kv_len, [1] pending token
    const int *page_table;               // logical page -> physical page
    uint16_t *kpool, *vpool;             // per (layer, page, head) a record of KV_PAGE*2*hd bf16, value = hi + lo:
                                         // K [position][term][hd], V [term][hd][position]
    const float2 *rope;                  // [max_ctx][hd/2] (cos, sin)
    const int *drafts;                   // device copy of this pass's drafts
    ee_verify_result *result;            // device address of the pinned result block
    int n_pages;
    int kv_len;                          // positions cached before this pass (host mirror of state[0])
    int pending;                         // token of row 0 (host mirror of state[1])
    int contig_base;                     // >= 0: logical page i is physical page contig_base + i (no table lookup needed)
};

struct Scratch {
    float *h;            // [rows_max][d]        residual stream
    float *q;            // [rows_max][d]        queries after RoPE (pair-interleaved inside each head)
    // GEMM inputs as two bf16 terms each (x = hi + lo up to ~16 mantissa bits), written by the
    // stage that produces them, k-tile-major: [k-tile][term][row of the pass][32]
    uint16_t *xn;        // [Kpad_d/32][2][rows][32]  gain * h for the next QKV or gate/up GEMM
    uint16_t *xh;        // [Kpad_d/32][2][head rows][32]  head_gain * (h, or h after the adapters) for the LM head; the rows
                         // of all exits that share one launch of the head, exit after exit
    uint16_t *attn;      // [Kpad_d/32][2][rows][32]  attention output
    uint16_t *u;         // [Kpad_F/32][2][rows][32]  silu(gate)*up
    uint16_t *xa;        // [Kpad_d/32][2][rows][32]  h itself: input of an exit head's adapters
    uint16_t *t;         // [Kpad_A/32][2][rows][32]  the adapters' hidden units after the activation
    float *ss_h;         // [nwg][rows_max]      partial sums of squares of the LM-head input's rows (head rows)
    float *ss_a;         // [nwg][rows_max]      partial sums of h^2 after the FFN block / embedding
    float *ss_f;         // [nwg][rows_max]      partial sums of h^2 after the attention block
    float *att_part;     // [items][ATT_ROWS][hd+2] attention partials (only when the position range is split)
    int *att_count;      // [units] items of the unit that have delivered their partials; zero between launches
    int *head_count;     // workgroups of a head launch that have delivered their candidates; zero between launches
    float *part;         // [K split][n-tile][rows][16] partial tiles of a launch whose K is split over workgroups
    int *part_count;     // [nwg] splits of a group of workgroups that have delivered their partial tiles; zero between launches
    float *logits;       // [heads][rows_max][V] when logits are kept
    int2 *cand;          // [nwg][rows_max]      per-workgroup argmax candidates (value bits, index)
    float *cand_sum;     // [nwg][rows_max]      sum over the workgroup's columns of exp(logit - candidate value)
};

enum HeadKind { HEAD_NONE = 0, HEAD_EXIT = 1, HEAD_FINAL = 2, HEAD_PREFILL = 3 };

// Probabilistic verification: inputs and per-row decisions.
struct SampleDev {
    const float *probs;  // [session][gamma][V]  the draft model's distributions
    const float *uv;     // per session 2 gamma + 2 floats: [gamma] the keep tests' uniform numbers, [gamma+1] the rows'
                         // sampling numbers, 1 / temperature
    int on;              // 1: the pass decides by the draft probabilities instead of by exact match
    int *tok;            // [head rows]  token a row emits if the round ends there
    int *kept;           // [head rows]  1: the row's draft passes its test
    int *count;          // rows of a sampling launch that have delivered; zero between launches
};

struct PassArgs {
    ModelDev mdv;                        // the model descriptor by value
    GemmPlan plan0;                      // plan, LDS map and weights of the launch's GEMM stage
    StageLds lay;
    const uint4 *W0;
    Scratch sc;
    int nwg;
    int n_sess, M, rows;                 // rows = n_sess * M
    int mode;                            // 0 verify, 1 prefill chunk
    const int *pf_tokens;                // prefill: [rows] token ids, < 0 => embedding row
    const uint16_t *pf_emb;              // prefill: [rows][d] bf16
    int pf_pos0;                         // prefill: position of row 0
    int layer_begin, layer_end;          // layers [begin, end) of this segment, 0-based
    int do_embed;
    int head_kind, head_idx;             // head_idx: result slot of the (first) head of this segment's head launch
    const float *head_gain;
    int n_heads;                         // exit heads evaluated by the head launch (their rows follow each other)
    int head_rows;                       // rows of the head launch: n_heads * rows
    int head_row0;                       // first head row this segment's exit writes (its position in the group)
    int head_stage;                      // 1: this segment ends with the head launch (else its exit only deposits its rows)
    int adapter;                         // 1: the exit has adapters (stages AD, AU between the last layer and the head)
    const float *ad_bdown, *ad_bup;      // adapter biases: [A] and [d] (the bottlenecks' output biases summed)
    int commit, keep_logits;
    int fuse_accept;                     // the head launch also runs the accept step (in the workgroup that finishes last)
    int att_splits;
    int H, d, Kpad_d;                    // copies of the model descriptor's fields for the attention kernel
    float att_scale;
    int stage;                           // index of this launch's stage in the segment's stage list
    const SessDev *sess;                 // device array [n_sess]
    SessDev sess0;                       // copy of sess[0]
    SampleDev sm;
};


}  // namespace ee
