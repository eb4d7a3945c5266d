// Structures shared by the host runtime and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ee.h"

namespace ee {

constexpr int WAVES_PER_WG = 8;          // 512 threads: two waves per SIMD
constexpr int WG_THREADS = WAVES_PER_WG * 64;
constexpr int KV_PAGE = 16;              // positions per KV page
constexpr int ATT_ROWS = 8;              // query rows handled together in attention
constexpr int ATT_MAX_SPLITS = 32;

// Tiled layout of one weight matrix W[N][K] (row-major in the model file).
// A tile is the A operand of one v_mfma_f32_16x16x32_bf16: 16 rows of N by 32
// columns of K, stored as 64 lanes x 16 bytes, lane l holding
// W[nt*16 + (l & 15)][kt*32 + (l >> 4)*8 .. +7].  Tiles are ordered
// [K-block][n-tile][k-tile inside the block]; a "run" is the KBT (or KBT_last)
// consecutive tiles of one (K-block, n-tile).  Wave w of NW streams the
// contiguous tile range [T*w/NW, T*(w+1)/NW) and emits one partial 16 x rows
// result per run it touches.
struct GemmPlan {
    int N, K;            // logical shape
    int NT, KT;          // tiles along N and K (zero padded)
    int KBT;             // k-tiles per full K-block
    int nKB;             // number of K-blocks
    int KBT_last;        // k-tiles in the last K-block
    int MAXP;            // most waves that share one run
    long long T;         // NT * KT
    float *part;         // partial results [nKB*NT runs][MAXP][rows_max][16]
};

struct LayerDev {
    const uint4 *wqkv, *wo, *wgu, *wd;   // tiled weights
    const float *g_attn, *g_ffn;         // norm gains
};

struct ModelDev {
    int L, d, H, hd, F, V;
    float eps, att_scale;
    int Kpad_d, Kpad_F;                  // K rounded up to 32
    int rows_max;
    GemmPlan qkv, o, gu, dn, head;
    const uint16_t *emb;                 // [V][d] bf16, row-major
    const uint4 *wlm;                    // tiled LM head
    const float *g_final;
    const LayerDev *layers;
};

struct SessDev {
    int *state;                          // [0] kv_len, [1] pending token
    const int *page_table;               // logical page -> physical page
    uint16_t *kpool, *vpool;             // [L][n_pages][H][KV_PAGE][hd] bf16
    const float2 *rope;                  // [max_ctx][hd/2] (cos, sin)
    const int *drafts;                   // device copy of this pass's drafts
    ee_verify_result *result;            // device address of the pinned result block
    int n_pages;
    int pad_;
};

struct GridBarrier {
    unsigned count;
    unsigned gen;
};

struct Scratch {
    float *h;            // [rows_max][d]        residual stream
    float *q;            // [rows_max][d]        queries after RoPE
    float *xn;           // [rows_max][Kpad_d]   gain-scaled hidden state, next GEMM input
    float *xh;           // [rows_max][Kpad_d]   same with the head's gain
    float *attn;         // [rows_max][Kpad_d]   attention output
    float *u;            // [rows_max][Kpad_F]   silu(gate)*up
    float *ss_a;         // [nwg][rows_max]      partial sums of h^2 after the FFN block / embedding
    float *ss_f;         // [nwg][rows_max]      partial sums of h^2 after the attention block
    float *att_part;     // attention partials
    float *logits;       // [heads][rows_max][V] when logits are kept
    int2 *cand;          // [nwg][rows_max]      per-workgroup argmax candidates (value bits, index)
    GridBarrier *bar;
    int *err;            // set to 1 when a bounded wait gave up
};

enum HeadKind { HEAD_NONE = 0, HEAD_EXIT = 1, HEAD_FINAL = 2, HEAD_PREFILL = 3 };

struct PassArgs {
    const ModelDev *md;
    Scratch sc;
    int nwg;
    int n_sess, M, rows;                 // rows = n_sess * M
    int mode;                            // 0 verify, 1 prefill chunk
    const int *pf_tokens;                // prefill: [rows] token ids, < 0 => embedding row
    const uint16_t *pf_emb;              // prefill: [rows][d] bf16
    int pf_pos0;                         // prefill: position of row 0
    int layer_begin, layer_end;          // layers [begin, end) of this segment, 0-based
    int do_embed;
    int head_kind, head_idx;
    const float *head_gain;
    int commit, keep_logits;
    int att_splits;
    int ph_lo, ph_hi;                    // window of this launch inside the segment's phase list
    unsigned spin_limit;
    const SessDev *sess;                 // device array [n_sess]
};

}  // namespace ee
