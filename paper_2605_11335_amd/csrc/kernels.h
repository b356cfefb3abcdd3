// Host-visible launchers of the block kernels.  Every launcher validates shapes against
// what its kernel assumes (`*_check` returns a message or nullptr) before anything runs.
#pragma once
#include "common.h"

enum { EPI_SPLIT_GELU = 0, EPI_GATE_RESID = 1 };

struct GemmArgs {
    const bf16* A;      // [M, lda] activations
    int lda;
    WView W;            // weight blob view
    uint64_t w_off;     // blob offset of W[0][0]; W is [N, K] bf16 row-major
    uint64_t bias_off;  // blob offset of bias[N] (bf16)
    int has_bias;
    int M, N, K;
    int n0, n1;         // output-feature panel covered by this launch
    int epi;
    // EPI_SPLIT_GELU: features [0, n_split) -> out0[m*ld0 + n] (bf16);
    //                 features [n_split, N) -> GELU -> out1[m*ld1 + col1_off + n - n_split]
    bf16* out0; int ld0; int n_split;
    bf16* out1; int ld1; int col1_off;
    int act_erf;        // the activation of out1: 0 = tanh form of GELU, 1 = erf form
    // EPI_GATE_RESID: y[m*ldy + n] = resid[m*ldy + n] + gate[n] * (acc + bias)   (fp32; gate NULL = 1)
    const float* resid; const float* gate; float* y; int ldy;
    // A batch of samples stacked along M (rows_per_sample > 0): row m is row i = m % rows_per_sample of
    // sample b = m / rows_per_sample; it uses gate + b*gate_bs and sits at b*resid_bs + i*ldy in resid,
    // b*y_bs + i*ldy in y (strides in elements).  rows_per_sample = 0: one sample, strides unused.
    int rows_per_sample; long gate_bs, resid_bs, y_bs;
};
const char* gemm_check(const GemmArgs& g);
int gemm_tile(const GemmArgs& g);      // tile gemm_launch will use: 0 = 256x256, 1 = 128x128
double gemm_fill(int M, int n);        // share of the launched rounds of workgroups that n features x M tokens fill
hipError_t gemm_launch(const GemmArgs& g, hipStream_t s);
hipError_t mfma_rate_launch(int iters, int random_operands, float* out, hipStream_t s);   // diagnostic: MFMAs on registers only
// diagnostic: MFMAs sharing the SIMD with LDS fragment reads and VALU work (see gemm.hip for the supported mixes)
hipError_t mix_rate_launch(int iters, int waves, int reads16, int valu, int exps, float* out, hipStream_t s);
// two independent problems in one launch; gemm_pair_tile: the tile shape they share (as gemm_tile), -1 = cannot pair
int gemm_pair_tile(const GemmArgs& g0, const GemmArgs& g1);
hipError_t gemm_launch_pair(const GemmArgs& g0, const GemmArgs& g1, hipStream_t s);

// Positions of this rank's tokens in the joint sequence: up to two contiguous segments
// (text rows, image rows).  Local row i < len0 sits at pos0 + i, else at pos1 + (i - len0).
struct TokenMap {
    int n_total, n_local;
    int pos0, len0, pos1, len1;
};

struct AttnArgs {
    const bf16* Q;      // [H, nq, hd] head-major
    const bf16* K;      // [H, nk, hd]
    const bf16* Vt;     // [H, hd, nk_pad] keys contiguous, pad columns zero
    bf16* O;            // element (h, q, :) at O + (h / hps)*o_bs + (h % hps)*o_hs + q*o_qs
    long o_hs, o_qs, o_bs;
    int H, nq, nk, nk_pad, hd;
    int hps;            // heads per sample (a batch is H / hps samples of hps heads each); 0 = H
    float scale;        // 1/sqrt(hd)
    // Scatter mode (the second Ulysses exchange, Sec. 2.1, done by the attention kernel's own stores; O unused):
    // query position q of head h (sample b = h / hps, head hh = h % hps) is one of this rank's positions in `map`
    // -> columns (h0 + hh)*hd of the output projection's operand, row i of the map's first segment at
    // dst0 + b*bs0 + i*ld, of its second segment at dst1 + b*bs1 + i*ld; any other position -> row of the send
    // buffer, send + b*send_bs + (hh*(n_total - n_local) + index among the remote positions)*hd (send NULL: dropped).
    int scatter;
    TokenMap map;
    bf16 *dst0, *dst1, *send;
    int ld, h0;
    long bs0, bs1, send_bs;
};
const char* attn_check(const AttnArgs& a);
hipError_t attn_launch(const AttnArgs& a, hipStream_t s);
int attn_waves(const AttnArgs& a);      // waves per workgroup attn_launch takes (host arithmetic only)

// m[b][n] = sum_k W[n,k] t[b][k] + bias[n]  (fp32 out), rows [n0, n1), for `batch` vectors t + b*K -> m + b*m_bs
hipError_t modvec_launch(const WView& W, uint64_t w_off, uint64_t b_off, const float* t, float* m,
                         int n0, int n1, int K, int batch, long m_bs, hipStream_t s);

// xn = LN(x) * (1 + scale) + shift  (fp32 in, bf16 out); with ln_w/ln_b (blob offsets, has_affine)
// instead: xn = LN(x) * w + b.
// Row r of a batch is row r % rows_per_sample of sample b = r / rows_per_sample: read at x + b*x_bs, modulated
// with shift + b*mod_bs, scale + b*mod_bs; written densely to xn + r*ld_out.
hipError_t ln_modulate_launch(const float* x, const float* shift, const float* scale, bf16* xn,
                              int rows, int d, int ld_out, int rows_per_sample, long x_bs, long mod_bs, hipStream_t s);
hipError_t ln_affine_launch(const float* x, const WView& W, uint64_t w_off, uint64_t b_off, bf16* xn,
                            int rows, int d, hipStream_t s);

// Split a projection output into head-major attention operands, with optional per-head RMSNorm.
struct RelayoutArgs {
    const bf16* src;        // [rows, ld] ; head h of tensor t at column col0[t] + h*hd
    int ld, rows;
    int col_q, col_k, col_v;          // -1 = tensor absent
    int n_heads;                      // heads present in src (H)
    int h0, h_local;                  // heads kept for attention: [h0, h0 + h_local)
    int hd;
    WView W; uint64_t qn_off, kn_off; int has_norm;
    const float *rope_cos, *rope_sin; // [n_local, hd/2] by local row, or NULL: rotate q,k pairs (2i, 2i+1) after the norm
    TokenMap map; int row0;           // src row i is local row row0 + i
    bf16 *Q, *K, *Vt;                 // [h_local, n_total, hd] x2, [h_local, hd, n_pad]
    int n_pad;
    bf16 *send_q, *send_k, *send_v;   // [n_heads - h_local, n_local, hd] (may be NULL)
};
hipError_t relayout_launch(const RelayoutArgs& r, hipStream_t s);

// What this rank receives from the second exchange (Sec. 2.1): the attention output of the other ranks' heads for
// its own tokens, peer_attn [n_local, n_heads - h_local, hd], copied into the columns of those heads in the
// output projection's operand (rows of the map's first segment at dst, of its second at dst1; leading dimension ld).
struct PeerAttnArgs {
    const bf16* peer_attn;            // NULL: nothing to copy
    bf16 *dst, *dst1;
    int ld, n_heads, h0, h_local, hd;
    TokenMap map;
};

// One launch for everything that does not depend on attention itself: the relayout of up to two parts (one per
// stream), when given the peer rows (what the first exchange delivers) placed at the remote positions of
// parts[0]'s operands (q, k copied; v transposed), and the peer attention rows of the second exchange.
hipError_t pre_attention_launch(const RelayoutArgs* parts, int n_parts, const bf16* peer_q, const bf16* peer_k,
                                const bf16* peer_v, const PeerAttnArgs& pa, hipStream_t s);

hipError_t checksum_launch(const void* data, uint64_t bytes, uint64_t first_word, uint64_t* out, hipStream_t s);
hipError_t f32_to_bf16_launch(const float* src, bf16* dst, size_t n, hipStream_t s);
