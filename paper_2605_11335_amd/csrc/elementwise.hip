// HBM-bound kernels of the block: adaLN modulation vector, LayerNorm+modulate, q/k RMSNorm
// with the Ulysses head-major relayout, the receiving side of the two exchanges around attention
// (Sec. 2.1; the sending side of the second one is the attention kernel's own stores), and the
// streamed-bytes checksum.  All accesses are 8- or 16-byte per lane and
// consecutive lanes touch consecutive addresses.
#include "common.h"
#include "kernels.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ void unpack8(const uint32x4& u, float* f) {
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
    f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
    f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
}
__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
    f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
    f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
}

__device__ __forceinline__ int local_pos(const TokenMap& m, int i) {
    return i < m.len0 ? m.pos0 + i : m.pos1 + (i - m.len0);
}
// i-th position (ascending) that is NOT local
__device__ __forceinline__ int remote_pos(const TokenMap& m, int i) {
    if (i < m.pos0) return i;
    i += m.len0;
    if (m.len1 == 0 || i < m.pos1) return i;
    return i + m.len1;
}

// ---------------------------------------------------------------------------------------------
// m[n] = W[n,:] . t + b[n]; a wave owns MV_ROWS consecutive rows so that each slice of t is read
// once per MV_ROWS weight vectors and that many 16-byte loads are in flight per lane.  A row's sum
// is accumulated in the same lane order whatever rows share its wave.
constexpr int MV_ROWS = 4;
// U steps of the walk over K are fetched together (U * (MV_ROWS + 2) loads in flight per lane): with one
// step per round trip to memory the kernel ran at the latency of K / 512 + MV_ROWS dependent loads, not
// at the bandwidth of the weight matrix.  A lane whose step lies past the end re-reads the row's last
// chunk and adds nothing.
template <int U>
__global__ __launch_bounds__(256) void modvec_kernel(WView W, uint64_t w_off, uint64_t b_off, const float* __restrict__ t,
                                                     float* __restrict__ m, int n0, int n1, int K, long m_bs) {
    t += (size_t)blockIdx.y * K;                 // one sample of the batch per grid row
    m += (size_t)blockIdx.y * m_bs;
    const int lane = threadIdx.x & 63;
    const int n = n0 + (blockIdx.x * 4 + (threadIdx.x >> 6)) * MV_ROWS;
    if (n >= n1) return;
    float acc[MV_ROWS];
#pragma unroll
    for (int r = 0; r < MV_ROWS; ++r) acc[r] = 0.f;
    const int nc = K / 8;                        // 16-byte chunks per row
    for (int c0 = lane; c0 < nc; c0 += 64 * U) {
        uint32x4 u[U][MV_ROWS];
        floatx4 t0[U], t1[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int c = min(c0 + 64 * q, nc - 1);
#pragma unroll
            for (int r = 0; r < MV_ROWS; ++r) {
                const int nr = min(n + r, n1 - 1);
                u[q][r] = *(const uint32x4*)wv_ptr(W, w_off + ((uint64_t)nr * K + (uint64_t)c * 8) * 2);
            }
            t0[q] = *(const floatx4*)(t + c * 8);
            t1[q] = *(const floatx4*)(t + c * 8 + 4);
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            if (c0 + 64 * q < nc) {
#pragma unroll
                for (int r = 0; r < MV_ROWS; ++r) {
                    float w[8];
                    unpack8(u[q][r], w);
                    acc[r] += w[0] * t0[q].x + w[1] * t0[q].y + w[2] * t0[q].z + w[3] * t0[q].w + w[4] * t1[q].x + w[5] * t1[q].y +
                              w[6] * t1[q].z + w[7] * t1[q].w;
                }
            }
        }
    }
    // lane r adds the bias of row r and writes it: the MV_ROWS bias loads go out side by side
    float mine = 0.f;
#pragma unroll
    for (int r = 0; r < MV_ROWS; ++r) {
        const float v = wave_sum(acc[r]);
        if (lane == r) mine = v;
    }
    if (lane < MV_ROWS && n + lane < n1) m[n + lane] = mine + wv_bf16(W, b_off, n + lane);
}

// ---------------------------------------------------------------------------------------------
// LayerNorm over d (no affine, biased variance, eps 1e-6) then modulate or affine; wave per row
template <int NJ, bool AFFINE>
__global__ __launch_bounds__(256) void ln_kernel(const float* __restrict__ x, const float* __restrict__ shift,
                                                 const float* __restrict__ scale, WView W, uint64_t w_off,
                                                 uint64_t b_off, bf16* __restrict__ out, int rows, int d, int ld_out,
                                                 int rows_per_sample, long x_bs, long mod_bs) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    // a batch stacks samples along the rows: each has its own modulation vectors and may sit at its own stride
    int smp = 0, ri = row;
    if (rows_per_sample) { smp = row / rows_per_sample; ri = row - smp * rows_per_sample; }
    const float* xr = x + (size_t)smp * x_bs + (size_t)ri * d;
    if (!AFFINE) { shift += (size_t)smp * mod_bs; scale += (size_t)smp * mod_bs; }
    float4 v[NJ];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        v[j] = *(const float4*)(xr + (lane + 64 * j) * 4);
        s += v[j].x + v[j].y + v[j].z + v[j].w;
    }
    // the row-independent operands of the last step are requested now, so that they arrive while the
    // statistics are reduced instead of costing a round trip of their own afterwards
    floatx4 ma[NJ], mb[NJ];                      // modulate: scale, shift;  affine: weight | bias as bf16 pairs
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int c = (lane + 64 * j) * 4;
        if (AFFINE) {
            const uint32x2 wa = *(const uint32x2*)wv_ptr(W, w_off + 2ull * c), wb = *(const uint32x2*)wv_ptr(W, b_off + 2ull * c);
            ma[j] = floatx4{__uint_as_float(wa.x << 16), __uint_as_float(wa.x & 0xffff0000u), __uint_as_float(wa.y << 16),
                            __uint_as_float(wa.y & 0xffff0000u)};
            mb[j] = floatx4{__uint_as_float(wb.x << 16), __uint_as_float(wb.x & 0xffff0000u), __uint_as_float(wb.y << 16),
                            __uint_as_float(wb.y & 0xffff0000u)};
        } else {
            ma[j] = *(const floatx4*)(scale + c);
            mb[j] = *(const floatx4*)(shift + c);
        }
    }
    const float mean = wave_sum(s) / d;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        v[j].x -= mean; v[j].y -= mean; v[j].z -= mean; v[j].w -= mean;
        q += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
    }
    const float rstd = rsqrtf(wave_sum(q) / d + 1e-6f);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int c = (lane + 64 * j) * 4;
        float a[4], b[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] = AFFINE ? ma[j][e] : 1.f + ma[j][e];
            b[e] = mb[j][e];
        }
        bf16x4 o;
        o[0] = (bf16)(v[j].x * rstd * a[0] + b[0]);
        o[1] = (bf16)(v[j].y * rstd * a[1] + b[1]);
        o[2] = (bf16)(v[j].z * rstd * a[2] + b[2]);
        o[3] = (bf16)(v[j].w * rstd * a[3] + b[3]);
        *(bf16x4*)(out + (size_t)row * ld_out + c) = o;
    }
}

template <bool AFFINE>
hipError_t ln_dispatch(const float* x, const float* shift, const float* scale, const WView& W, uint64_t w_off,
                       uint64_t b_off, bf16* out, int rows, int d, int ld_out, int rows_per_sample, long x_bs, long mod_bs,
                       hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    if (d % 256 || d > 4096 || rows_per_sample < 0 || (x_bs % 4) || (mod_bs % 4)) return hipErrorInvalidValue;
    const dim3 grid((rows + 3) / 4), blk(256);
#define CF_LN_CASE(NJ) case NJ: hipLaunchKernelGGL((ln_kernel<NJ, AFFINE>), grid, blk, 0, s, x, shift, scale, W, w_off, b_off, out, rows, d, ld_out, rows_per_sample, x_bs, mod_bs); break;
    switch (d / 256) {
        CF_LN_CASE(1) CF_LN_CASE(2) CF_LN_CASE(3) CF_LN_CASE(4) CF_LN_CASE(6) CF_LN_CASE(8) CF_LN_CASE(12) CF_LN_CASE(16)
        default: return hipErrorInvalidValue;
    }
#undef CF_LN_CASE
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// q,k: optional per-head RMSNorm, then head-major placement (own heads) or send buffers (others).
// v of other heads: send buffer.  A group of hd/8 lanes owns one (row, tensor, head) vector.
__device__ __forceinline__ void qk_relayout_part(const RelayoutArgs& r, int bid, int nblk) {
    const int lph = r.hd / 8;                       // lanes per head vector
    const int vec_per_blk = 256 / lph;
    const long n_vec = (long)r.rows * 3 * r.n_heads;
    const int sub = threadIdx.x % lph;
    for (long vi = (long)bid * vec_per_blk + threadIdx.x / lph; vi < n_vec; vi += (long)nblk * vec_per_blk) {
        const int hh = vi % r.n_heads;
        const int tns = (vi / r.n_heads) % 3;       // 0 q, 1 k, 2 v
        const int row = vi / (3 * r.n_heads);
        const int col = tns == 0 ? r.col_q : (tns == 1 ? r.col_k : r.col_v);
        const bool own = hh >= r.h0 && hh < r.h0 + r.h_local;
        bf16* dst;
        const int lrow = r.row0 + row;
        if (own) {
            if (tns == 2) continue;                 // own v goes through the transposing kernel
            bf16* base = tns == 0 ? r.Q : r.K;
            dst = base + ((size_t)(hh - r.h0) * r.map.n_total + local_pos(r.map, lrow)) * r.hd;
        } else {
            bf16* base = tns == 0 ? r.send_q : (tns == 1 ? r.send_k : r.send_v);
            if (!base) continue;
            const int ho = hh < r.h0 ? hh : hh - r.h_local;
            dst = base + ((size_t)ho * r.map.n_local + lrow) * r.hd;
        }
        if (col < 0) continue;
        uint4 u = *(const uint4*)(r.src + (size_t)row * r.ld + col + hh * r.hd + sub * 8);
        if ((r.has_norm || r.rope_cos) && tns < 2) {
            float f[8];
            unpack8(u, f);
            if (r.has_norm) {
                float ss = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
                for (int o = lph >> 1; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
                const float rs = rsqrtf(ss / r.hd + 1e-6f);
                const uint4 wu = *(const uint4*)wv_ptr(r.W, (tns == 0 ? r.qn_off : r.kn_off) + sub * 16);
                float w[8];
                unpack8(wu, w);
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] = f[e] * rs * w[e];
            }
            if (r.rope_cos) {
                // this lane's 8 elements are pairs sub*4 .. sub*4+3 of the head vector
                const size_t ro = (size_t)lrow * (r.hd / 2) + sub * 4;
                const float4 cs = *(const float4*)(r.rope_cos + ro), sn = *(const float4*)(r.rope_sin + ro);
                const float c[4] = {cs.x, cs.y, cs.z, cs.w}, s4[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = f[2 * e], b = f[2 * e + 1];
                    f[2 * e] = a * c[e] - b * s4[e];
                    f[2 * e + 1] = a * s4[e] + b * c[e];
                }
            }
            bf16x8 o8;
#pragma unroll
            for (int e = 0; e < 8; ++e) o8[e] = (bf16)f[e];
            *(bf16x8*)(dst + sub * 8) = o8;
        } else {
            *(uint4*)(dst + sub * 8) = u;
        }
    }
}

// [token, hd] rows of one head -> Vt[head, d, position] (keys contiguous).  64 tokens per block.
// src element (h, i, d) at src + h*src_hs + i*src_rs + d; i counts local rows (remote=0) or
// remote rows (remote=1) and maps to its position in the joint sequence.
__device__ __forceinline__ void v_transpose_part(uint16_t* tile, int bx, int h, const bf16* __restrict__ src, long src_hs,
                                                 long src_rs, int n_rows, int row0, bf16* __restrict__ Vt, int hd, int n_pad,
                                                 const TokenMap& map, int remote) {
    const int i0 = bx * 64;
    const int stride = hd + 2;
    const int cpr = hd / 8;
    for (int q = threadIdx.x; q < 64 * cpr; q += 256) {
        const int tr = q / cpr, c = q % cpr;
        uint4 u = make_uint4(0, 0, 0, 0);
        if (i0 + tr < n_rows) u = *(const uint4*)(src + (size_t)h * src_hs + (size_t)(i0 + tr) * src_rs + c * 8);
        uint32_t* t32 = (uint32_t*)(tile + tr * stride + c * 8);   // stride even: 4-byte aligned
        t32[0] = u.x; t32[1] = u.y; t32[2] = u.z; t32[3] = u.w;
    }
    __syncthreads();
    // each thread: one d row, 8 consecutive tokens
    for (int q = threadIdx.x; q < hd * 8; q += 256) {
        const int dd = q >> 3, tg = (q & 7) * 8;
        if (i0 + tg >= n_rows) continue;
        const int i_first = row0 + i0 + tg;
        const int p_first = remote ? remote_pos(map, i_first) : local_pos(map, i_first);
        const int cnt = min(8, n_rows - (i0 + tg));
        const int i_last = i_first + cnt - 1;
        const int p_last = remote ? remote_pos(map, i_last) : local_pos(map, i_last);
        bf16* drow = Vt + ((size_t)h * hd + dd) * n_pad;
        if (cnt == 8 && p_last - p_first == 7 && (p_first & 7) == 0) {
            uint16_t e[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) e[k] = tile[(tg + k) * stride + dd];
            uint4 u;
            u.x = e[0] | ((uint32_t)e[1] << 16); u.y = e[2] | ((uint32_t)e[3] << 16);
            u.z = e[4] | ((uint32_t)e[5] << 16); u.w = e[6] | ((uint32_t)e[7] << 16);
            *(uint4*)(drow + p_first) = u;
        } else {
            for (int k = 0; k < cnt; ++k) {
                const int p = remote ? remote_pos(map, i_first + k) : local_pos(map, i_first + k);
                ((uint16_t*)drow)[p] = tile[(tg + k) * stride + dd];
            }
        }
    }
    // zero the pad columns once per (head, d) row
    if (bx == 0 && !remote) {
        for (int q = threadIdx.x; q < hd * (n_pad - map.n_total); q += 256) {
            const int dd = q / (n_pad - map.n_total), p = map.n_total + q % (n_pad - map.n_total);
            ((uint16_t*)Vt)[((size_t)h * hd + dd) * n_pad + p] = 0;
        }
    }
}

// peer q/k rows -> head-major operands at the remote positions (16-byte chunk copies)
__device__ __forceinline__ void peer_qk_part(int bid, int nblk, const bf16* __restrict__ pq, const bf16* __restrict__ pk,
                                             bf16* __restrict__ Q, bf16* __restrict__ K, int h_local, int hd, const TokenMap& map) {
    const int cpr = hd / 8;
    const int n_rem = map.n_total - map.n_local;
    const long total = 2L * h_local * n_rem * cpr;
    for (long q = (long)bid * 256 + threadIdx.x; q < total; q += (long)nblk * 256) {
        const int c = q % cpr;
        long rest = q / cpr;
        const int i = rest % n_rem; rest /= n_rem;
        const int h = rest % h_local;
        const int tns = rest / h_local;
        const bf16* s = (tns ? pk : pq) + ((size_t)h * n_rem + i) * hd + c * 8;
        bf16* d = (tns ? K : Q) + ((size_t)h * map.n_total + remote_pos(map, i)) * hd + c * 8;
        *(uint4*)d = *(const uint4*)s;
    }
}

// attention rows of the other ranks' heads for this rank's tokens -> their columns of the projection operand
__device__ __forceinline__ void peer_attn_part(int bid, int nblk, const PeerAttnArgs& p) {
    const int cpr = p.hd / 8, n_other = p.n_heads - p.h_local;
    const long total = (long)p.map.n_local * n_other * cpr;
    for (long q = (long)bid * 256 + threadIdx.x; q < total; q += (long)nblk * 256) {
        const int c = q % cpr;
        long rest = q / cpr;
        const int ho = rest % n_other;
        const int i = rest / n_other;
        const int hh = ho < p.h0 ? ho : ho + p.h_local;
        bf16* row = i < p.map.len0 ? p.dst + (size_t)i * p.ld : p.dst1 + (size_t)(i - p.map.len0) * p.ld;
        *(uint4*)(row + hh * p.hd + c * 8) = *(const uint4*)(p.peer_attn + ((size_t)i * n_other + ho) * p.hd + c * 8);
    }
}

// Everything between the QKV projection and attention in ONE launch: per part (one per stream)
// the q/k RMSNorm + head-major relayout and the transposition of the own heads' v, then the peer
// rows (q, k copied, v transposed).  Workgroups are dealt to the sub-tasks by index range.
struct PreAttnArgs {
    RelayoutArgs part[2];
    int n_parts;
    const bf16 *peer_q, *peer_k, *peer_v;      // may be NULL (sp_degree 1, or projection-only use)
    PeerAttnArgs pa;
    int seg[7];                                // end of each segment: qk0, vt0, qk1, vt1, peer_qk, peer_vt, peer_attn
};

__global__ __launch_bounds__(256) void pre_attention_kernel(PreAttnArgs a) {
    __shared__ uint16_t tile[64 * (128 + 2)];
    const int b = blockIdx.x;
    int lo = 0;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        if (p >= a.n_parts) break;
        const RelayoutArgs& r = a.part[p];
        if (b < a.seg[2 * p]) { qk_relayout_part(r, b - lo, a.seg[2 * p] - lo); return; }
        lo = a.seg[2 * p];
        if (b < a.seg[2 * p + 1]) {
            const int nbx = (r.rows + 63) / 64, i = b - lo;
            v_transpose_part(tile, i % nbx, i / nbx, r.src + r.col_v + (size_t)r.h0 * r.hd, (long)r.hd, (long)r.ld, r.rows,
                             r.row0, r.Vt, r.hd, r.n_pad, r.map, 0);
            return;
        }
        lo = a.seg[2 * p + 1];
    }
    const RelayoutArgs& r0 = a.part[0];
    const int n_rem = r0.map.n_total - r0.map.n_local;
    if (b < a.seg[4]) { peer_qk_part(b - lo, a.seg[4] - lo, a.peer_q, a.peer_k, r0.Q, r0.K, r0.h_local, r0.hd, r0.map); return; }
    lo = a.seg[4];
    if (b < a.seg[5]) {
        const int nbx = (n_rem + 63) / 64, i = b - lo;
        v_transpose_part(tile, i % nbx, i / nbx, a.peer_v, (long)n_rem * r0.hd, (long)r0.hd, n_rem, 0, r0.Vt, r0.hd, r0.n_pad,
                         r0.map, 1);
        return;
    }
    lo = a.seg[5];
    if (b < a.seg[6]) peer_attn_part(b - lo, a.seg[6] - lo, a.pa);
}

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zero_u64_kernel(uint64_t* p) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0; }

// sum over 64-bit words of mix(word ^ (index+1)*GOLDEN), index counted from the blob start
__global__ __launch_bounds__(256) void checksum_kernel(const uint64_t* __restrict__ w, uint64_t n_words, uint64_t first_word,
                                                       unsigned long long* __restrict__ out) {
    uint64_t acc = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n_words; i += (uint64_t)gridDim.x * 256)
        acc += cf_mix64(w[i] ^ ((first_word + i + 1) * CF_GOLDEN64));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)acc, o), hi = __shfl_xor((uint32_t)(acc >> 32), o);
        acc += ((uint64_t)hi << 32) | lo;
    }
    if ((threadIdx.x & 63) == 0) atomicAdd(out, (unsigned long long)acc);
}

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ s, bf16* __restrict__ d, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) d[i] = (bf16)s[i];
}

inline int grid_for(long items, int per_block, int cap = 256 * 16) {
    long b = (items + per_block - 1) / per_block;
    return (int)(b < 1 ? 1 : (b > cap ? cap : b));
}

}  // namespace

hipError_t modvec_launch(const WView& W, uint64_t w_off, uint64_t b_off, const float* t, float* m, int n0, int n1,
                         int K, int batch, long m_bs, hipStream_t s) {
    if (n1 <= n0) return hipSuccess;
    if (K % 8 || batch < 1 || batch > 65535) return hipErrorInvalidValue;
    const dim3 grid((n1 - n0 + 4 * MV_ROWS - 1) / (4 * MV_ROWS), batch);
    const int steps = (K / 8 + 63) / 64;         // steps of a lane's walk over K; taken 3 or 4 at a time
#define CF_MV_CASE(U) hipLaunchKernelGGL(modvec_kernel<U>, grid, dim3(256), 0, s, W, w_off, b_off, t, m, n0, n1, K, m_bs)
    if (steps == 1) CF_MV_CASE(1);
    else if (steps == 2) CF_MV_CASE(2);
    else if (steps % 3 == 0) CF_MV_CASE(3);
    else CF_MV_CASE(4);
#undef CF_MV_CASE
    return hipGetLastError();
}

hipError_t ln_modulate_launch(const float* x, const float* shift, const float* scale, bf16* xn, int rows, int d,
                              int ld_out, int rows_per_sample, long x_bs, long mod_bs, hipStream_t s) {
    WView none{nullptr, nullptr, 0};
    return ln_dispatch<false>(x, shift, scale, none, 0, 0, xn, rows, d, ld_out, rows_per_sample, x_bs, mod_bs, s);
}

hipError_t ln_affine_launch(const float* x, const WView& W, uint64_t w_off, uint64_t b_off, bf16* xn, int rows, int d,
                            hipStream_t s) {
    return ln_dispatch<true>(x, nullptr, nullptr, W, w_off, b_off, xn, rows, d, d, 0, 0, 0, s);
}

hipError_t pre_attention_launch(const RelayoutArgs* parts, int n_parts, const bf16* peer_q, const bf16* peer_k,
                                const bf16* peer_v, const PeerAttnArgs& pa, hipStream_t s) {
    if (n_parts < 1 || n_parts > 2) return hipErrorInvalidValue;
    PreAttnArgs a{};
    a.n_parts = n_parts;
    a.peer_q = peer_q; a.peer_k = peer_k; a.peer_v = peer_v;
    a.pa = pa;
    int end = 0;
    for (int p = 0; p < 2; ++p) {
        if (p < n_parts) {
            const RelayoutArgs& r = parts[p];
            if (r.hd != 64 && r.hd != 128) return hipErrorInvalidValue;
            a.part[p] = r;
            if (r.rows > 0) end += grid_for((long)r.rows * 3 * r.n_heads, 256 / (r.hd / 8));
            a.seg[2 * p] = end;
            if (r.rows > 0 && r.col_v >= 0 && r.Vt) end += ((r.rows + 63) / 64) * r.h_local;
            a.seg[2 * p + 1] = end;
        } else {
            a.seg[2 * p] = a.seg[2 * p + 1] = end;
        }
    }
    const RelayoutArgs& r0 = parts[0];
    const int n_rem = r0.map.n_total - r0.map.n_local;
    if (peer_q && peer_k && peer_v && n_rem > 0) {
        end += grid_for(2L * r0.h_local * n_rem * (r0.hd / 8), 256);
        a.seg[4] = end;
        end += ((n_rem + 63) / 64) * r0.h_local;
        a.seg[5] = end;
    } else {
        a.seg[4] = a.seg[5] = end;
    }
    if (pa.peer_attn && pa.n_heads > pa.h_local && pa.map.n_local > 0) {
        if ((pa.hd != 64 && pa.hd != 128) || !pa.dst || (pa.ld % 8)) return hipErrorInvalidValue;
        if (!a.pa.dst1) a.pa.dst1 = pa.dst + (size_t)pa.map.len0 * pa.ld;
        end += grid_for((long)pa.map.n_local * (pa.n_heads - pa.h_local) * (pa.hd / 8), 256);
    }
    a.seg[6] = end;
    if (end == 0) return hipSuccess;
    hipLaunchKernelGGL(pre_attention_kernel, dim3(end), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t relayout_launch(const RelayoutArgs& r, hipStream_t s) {
    return pre_attention_launch(&r, 1, nullptr, nullptr, nullptr, PeerAttnArgs{}, s);
}

hipError_t checksum_launch(const void* data, uint64_t bytes, uint64_t first_word, uint64_t* out, hipStream_t s) {
    if (bytes % 8 || ((uintptr_t)data % 8)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(64), 0, s, out);
    if (bytes)
        hipLaunchKernelGGL(checksum_kernel, dim3(grid_for((long)(bytes / 8), 256 * 8, 2048)), dim3(256), 0, s,
                           (const uint64_t*)data, bytes / 8, first_word, (unsigned long long*)out);
    return hipGetLastError();
}

hipError_t f32_to_bf16_launch(const float* src, bf16* dst, size_t n, hipStream_t s) {
    if (!n) return hipSuccess;
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(grid_for((long)n, 256 * 4)), dim3(256), 0, s, src, dst, n);
    return hipGetLastError();
}
