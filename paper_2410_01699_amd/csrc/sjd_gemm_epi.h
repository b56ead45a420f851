// Pieces shared by the two bf16 projection kernels (the skinny one for up to 32 rows and the wide one for
// up to 128): MFMA operand types, the hi / lo split, and the epilogues that see final fp32 sums (plain
// store, residual add + operands of the next normalisation, SiLU(gate) * up, RoPE + KV-cache write;
// paper Sec. 4.1 Step 2).  Included by those two files only.
#pragma once
#include "sjd_internal.h"

// what a projection does with its activations before the product
#define SJD_PRO_PLAIN 0     // fp32 activations as they are
#define SJD_PRO_NORM 1      // planes of x * gain; the token factors rsqrt(mean(x^2) + eps) come from partial sums
#define SJD_PRO_A24 2       // activations in hi / lo planes, as they are
#define SJD_PRO_NORM16 3    // as SJD_PRO_NORM, the lo plane in its 2-byte form (the second operand ready made)
#define SJD_PRO_A16 4       // as SJD_PRO_A24, the lo plane in its 2-byte form

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// hi = bf16(x) (round to nearest even), lo = bf16(x - hi)
__device__ __forceinline__ void split8(const float (&x)[8], bf16x8 &hi, bf16x8 &lo)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const __bf16 h = (__bf16)x[e];
        hi[e] = h;
        lo[e] = (__bf16)(x[e] - (float)h);
    }
}

// second operand of 8 values from their hi plane entry (8 bf16) and their byte plane entry (8 bytes):
// value = hi bits | lo byte << 8 (as fp32); second operand = bf16(value - hi), exact
__device__ __forceinline__ bf16x8 lo_from_byte_plane(bf16x8 hi, uint2 lo8)
{
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const u32x4 hw = __builtin_bit_cast(u32x4, hi);
    bf16x8 lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t hw_ = hw[e >> 1], lw_ = (e < 4) ? lo8.x : lo8.y;
        const uint32_t hb_ = (e & 1) ? (hw_ & 0xFFFF0000u) : (hw_ << 16);
        const uint32_t lb_ = ((lw_ >> (8 * (e & 3))) & 0xFFu) << 8;
        lo[e] = (__bf16)(__uint_as_float(hb_ | lb_) - __uint_as_float(hb_));
    }
    return lo;
}

__device__ __forceinline__ uint32_t pack_hi2(float a, float b, float &ra, float &rb)
{
    const bf16_t ha = f32_to_bf16(a), hb = f32_to_bf16(b);
    ra = a - bf16_to_f32(ha); rb = b - bf16_to_f32(hb);
    return (uint32_t)ha | ((uint32_t)hb << 16);
}

// What an epilogue needs from memory besides the sums; fetched while the weights stream.
struct EpiPre {
    f32x4 x;                  // RESID: current residual values
    uint2 gn;                 // RESID: 4 bf16 gains of the normalisation that follows
    float c0, s0, c1, s1;     // QKV: RoPE factors of this thread's two pairs
    int pos;                  // QKV: absolute position of row m in its stream's cache
    int row;                  // QKV: row index inside the stream
    bf16_t *cache;            // QKV: this layer of the stream's cache (NULL: the row belongs to no stream)
};

template <int EPI>
__device__ __forceinline__ void preload_epilogue(const SjdGemmEpi &ep, int N, int m, int n0, EpiPre &pre)
{
    if (EPI == SJD_EPI_RESID) {
        pre.x = *reinterpret_cast<const f32x4 *>(ep.out + act_off(m, n0, N / 32));
        pre.gn = ep.out24 ? *reinterpret_cast<const uint2 *>(ep.gain_next + n0) : make_uint2(0u, 0u);
    } else if (EPI == SJD_EPI_QKV) {
        const int half = ep.hd >> 1;
        // the stream that owns row m: its cache length and cache (the loop index is uniform, so the
        // table reads are scalar loads; the selection is per lane)
        const int stream = m >> ep.sm.shift;
        pre.row = m & ((1 << ep.sm.shift) - 1);
        int n_s = ep.sm.count > 0 ? *ep.sm.first.n : 0;
        pre.cache = (stream == 0 && ep.sm.count > 0) ? ep.sm.first.kvc + ep.layer_off : nullptr;
        for (int s = 1; s < ep.sm.count; ++s) {            // uniform index: scalar table reads
            const SjdStreamEntry e = ep.sm.table[s];
            const int n_here = *e.n;
            if (s == stream) { n_s = n_here; pre.cache = e.kvc + ep.layer_off; }
        }
        pre.pos = min(n_s + pre.row, ep.max_seq - 1);   // rows past the window are computed but never stored
        // (V fragments fetch factors they do not use: no branch around the loads)
        const int j = ((n0 % ep.d) % ep.hd) >> 1;
        const float2 cc = *reinterpret_cast<const float2 *>(ep.cosT + (size_t)pre.pos * half + j);
        const float2 ss = *reinterpret_cast<const float2 *>(ep.sinT + (size_t)pre.pos * half + j);
        pre.c0 = cc.x; pre.c1 = cc.y; pre.s0 = ss.x; pre.s1 = ss.y;
    }
}

// One accumulator fragment: lane l of the MFMA result holds features n0..n0+3 (packed order) of
// token m.  v = final sums.
template <int EPI>
__device__ __forceinline__ void apply_epilogue(const SjdGemmEpi &ep, int N, int m, int n0, f32x4 v, const EpiPre &pre)
{
    if (EPI == SJD_EPI_STORE) {
        *reinterpret_cast<f32x4 *>(ep.out + (size_t)m * N + n0) = v;
    } else if (EPI == SJD_EPI_RESID) {
        const f32x4 y = pre.x + v;
        *reinterpret_cast<f32x4 *>(ep.out + act_off(m, n0, N / 32)) = y;
        if (ep.out24) {
            // what the projection behind the next normalisation reads: x * gain in planes, and this
            // tile's share of sum(x^2) of token m (lanes l, l^16, l^32, l^48 hold its 16 features)
            act24_store4(ep.out24, m, n0, N / 32, y[0] * __uint_as_float(pre.gn.x << 16),
                         y[1] * __uint_as_float(pre.gn.x & 0xFFFF0000u), y[2] * __uint_as_float(pre.gn.y << 16),
                         y[3] * __uint_as_float(pre.gn.y & 0xFFFF0000u), ep.lo16 != 0);
            float sq = fmaf(y[0], y[0], fmaf(y[1], y[1], fmaf(y[2], y[2], y[3] * y[3])));
            sq += __shfl_xor(sq, 16);
            sq += __shfl_xor(sq, 32);
            if ((threadIdx.x & 48) == 0) ep.ssq_out[(size_t)m * ssq_stride(N) + (n0 >> 4)] = sq;
        }
    } else if (EPI == SJD_EPI_SILU) {
        // packed rows: (gate f, up f, gate f+1, up f+1)
        const int f = n0 >> 1;
        act24_store2(ep.ffn, m, f, ep.F / 32, v[0] / (1.0f + __expf(-v[0])) * v[1], v[2] / (1.0f + __expf(-v[2])) * v[3], ep.lo16 != 0);
    } else {   // SJD_EPI_QKV
        const int d = ep.d, hd = ep.hd, half = hd >> 1;
        const int pos = pre.pos;
        if (n0 < 2 * d) {
            // Q or K: packed order inside a head is (j, j+half, j+1, j+1+half, ...)
            const int is_k = n0 >= d;
            const int c = n0 - (is_k ? d : 0);
            const int head = c / hd, j = (c % hd) >> 1;
            const float c0 = pre.c0, s0 = pre.s0, c1 = pre.c1, s1 = pre.s1;
            const float r0 = v[0] * c0 - v[1] * s0, r0p = v[1] * c0 + v[0] * s0;   // dims j, j+half
            const float r1 = v[2] * c1 - v[3] * s1, r1p = v[3] * c1 + v[2] * s1;   // dims j+1, j+1+half
            if (!is_k) {
                float *q = ep.qact + (size_t)m * d + head * hd + j;
                *reinterpret_cast<float2 *>(q) = make_float2(r0, r1);
                *reinterpret_cast<float2 *>(q + half) = make_float2(r0p, r1p);
            } else if (pre.row < ep.rows_valid && pre.cache) {
                bf16_t *rec = pre.cache + kv_block_off(head, pos >> 5, ep.nblk, hd);
                const int kk = pos & 31;
                float la, lb, dummy0, dummy1;
                uint32_t hi = pack_hi2(r0, r1, la, lb);
                *reinterpret_cast<uint32_t *>(rec + kv_k_off(kk, j, hd, 0)) = hi;
                *reinterpret_cast<uint32_t *>(rec + kv_k_off(kk, j, hd, 1)) = pack_hi2(la, lb, dummy0, dummy1);
                hi = pack_hi2(r0p, r1p, la, lb);
                *reinterpret_cast<uint32_t *>(rec + kv_k_off(kk, j + half, hd, 0)) = hi;
                *reinterpret_cast<uint32_t *>(rec + kv_k_off(kk, j + half, hd, 1)) = pack_hi2(la, lb, dummy0, dummy1);
            }
        } else if (pre.row < ep.rows_valid && pre.cache) {
            // V: natural feature order
            const int col = n0 - 2 * d;
            const int head = col / hd, dim = col % hd;
            bf16_t *rec = pre.cache + kv_block_off(head, pos >> 5, ep.nblk, hd);
            const int kk = pos & 31;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bf16_t h = f32_to_bf16(v[r]);
                rec[kv_v_off(kk, dim + r, hd, 0)] = h;
                rec[kv_v_off(kk, dim + r, hd, 1)] = f32_to_bf16(v[r] - bf16_to_f32(h));
            }
        }
    }
}

