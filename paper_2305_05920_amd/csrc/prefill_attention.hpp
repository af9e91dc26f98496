// Initialization-phase (prompt) attention for gfx950: every token of a job's prompt attends
// to the tokens of the same prompt up to and including itself (FastServe, Section 2.2 and
// Figure 3: the first iteration of a job processes all its input tokens at once).
//
// Included by fastserve.hip inside its unnamed namespace; uses its element-type tags and
// small helpers.  This is the one dense contraction of the method, so it runs on the
// matrix cores (v_mfma_f32_32x32x16 with bf16 or f16 operands, fp32 accumulation).
//
// Work split.  A workgroup of 4 waves owns 128 consecutive query rows of one (job, head);
// wave w owns rows [32w, 32w+32) of them.  Keys and values of the pair are walked in
// tiles of 64 tokens, staged once per workgroup in LDS: keys as they lie in memory
// ([key][d], rows padded by 16 B), values transposed ([d][key], rows padded by 16 B), so
// that both matrix-core operands are plain 16-byte (keys) or 8-byte (values) LDS reads.
//
// Per tile a wave computes the transposed score tile S^T = K Q^T (keys x query rows): in
// the accumulator layout of the 32x32 instruction a lane then holds 16 keys of ONE query
// row (row = lane % 32, the other 16 keys sit in lane ^ 32), so the softmax statistics
// are per-lane scalars and need one exchange between the two half-waves.  The same
// registers, rounded to the storage type, are exactly the B operand of O^T = V^T P^T for
// the key order k = 8*(e/4) + 4*(lane/32) + e%4, which the reads of V^T follow; no
// cross-lane movement of the probabilities is needed.
#pragma once

constexpr int kPfQTile = 128;  // query rows per workgroup
constexpr int kPfKTile = 64;   // keys staged per iteration

typedef __bf16 pf_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 pf_f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 pf_bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 pf_f16x2 __attribute__((ext_vector_type(2)));
typedef float pf_f32x16 __attribute__((ext_vector_type(16)));
typedef float pf_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t pf_u32x2 __attribute__((ext_vector_type(2)));

template <typename E>
struct PfMath;
template <>
struct PfMath<BF16> {
    static __device__ __forceinline__ pf_f32x16 mfma(u32x4 a, u32x4 b, pf_f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pf_bf16x8, a),
                                                       __builtin_bit_cast(pf_bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        pf_bf16x2 r = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, r);
    }
};
template <>
struct PfMath<F16> {
    static __device__ __forceinline__ pf_f32x16 mfma(u32x4 a, u32x4 b, pf_f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(pf_f16x8, a),
                                                      __builtin_bit_cast(pf_f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        pf_f16x2 r = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(uint32_t, r);
    }
};

// q, k, v: [total_tokens][H][D] (2-byte elements), jobs packed back to back; offs[J+1].
// out: [total_tokens][H][D] fp32.  Grid: num_qtiles * pairs_padded workgroups; workgroup b
// serves pair b % pairs_padded (pairs_padded is a multiple of 8, so all tiles of a pair
// land on the same die and share its L2) and query tile num_qtiles-1 - b/pairs_padded
// (the tiles with the most keys start first).
template <typename E, int D>
__global__ __launch_bounds__(kThreads, 2) void fs_prefill_attn_kernel(
    const char *__restrict__ q, const char *__restrict__ k, const char *__restrict__ v,
    const int32_t *__restrict__ offs, float *__restrict__ out, int32_t J, int32_t H, int32_t pairs_padded,
    int32_t num_qtiles, long long total_tokens, float scale_log2e, int32_t *__restrict__ err)
{
    constexpr int kKStride = D * 2 + 16;         // bytes per staged key row
    constexpr int kVStride = kPfKTile * 2 + 16;  // bytes per staged row of V^T
    constexpr int NC = D / 16;                   // 16-wide chunks of the head dimension
    constexpr int ND = D / 32;                   // 32-wide tiles of the output's head dimension
    constexpr int kKChunks = D / 8;              // 16-byte chunks per key row
    constexpr int kKRowsPerPass = kThreads / kKChunks;
    constexpr int KP = kPfKTile / kKRowsPerPass;  // key-staging passes
    constexpr int VP = kKChunks / 8;              // value-staging passes (8 chunks per pass)
    __shared__ __attribute__((aligned(16))) char ks[kPfKTile * kKStride];
    __shared__ __attribute__((aligned(16))) char vt[D * kVStride];

    const int b = blockIdx.x;
    const int pair = b % pairs_padded;
    const int qt = num_qtiles - 1 - b / pairs_padded;
    if (pair >= J * H) return;
    const int j = pair / H, h = pair - j * H;
    const long long t0 = offs[j], t1 = offs[j + 1];
    if (t0 < 0 || t1 < t0 || t1 > total_tokens) {
        if (threadIdx.x == 0 && h == 0 && qt == 0) atomicOr(err, kErrBadLen);
        return;
    }
    const int s = (int)(t1 - t0);
    if (s > num_qtiles * kPfQTile) {  // longer than the launch was sized for
        if (threadIdx.x == 0 && h == 0 && qt == 0) atomicOr(err, kErrBadLen);
        return;
    }
    if (qt * kPfQTile >= s) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, hh = lane >> 5;
    const int row0 = qt * kPfQTile + wave * 32;  // first query row of this wave
    const int qrow = row0 + r;                   // this lane's query row (may lie past the prompt)
    const size_t tok_bytes = (size_t)H * D * 2;
    const size_t head_off = (size_t)h * D * 2;
    const char *kb = k + (size_t)t0 * tok_bytes + head_off;
    const char *vb = v + (size_t)t0 * tok_bytes + head_off;

    // Q^T operand: this lane's query row, the 8 elements d = 16c + 8*hh .. +8 of every chunk
    u32x4 qf[NC];
    {
        const char *qb = q + ((size_t)t0 + (size_t)(qrow < s ? qrow : s - 1)) * tok_bytes + head_off;
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[c] = *(const u32x4 *)(qb + c * 32 + hh * 16);
    }

    const int last_row = (qt * kPfQTile + kPfQTile < s ? qt * kPfQTile + kPfQTile : s) - 1;
    const int nkt = last_row / kPfKTile + 1;

    // staging roles of this thread
    const int k_row = threadIdx.x / kKChunks, k_chunk = threadIdx.x % kKChunks;
    const int v_pair = threadIdx.x & 31, v_chunk = threadIdx.x >> 5;  // keys 2*v_pair, 2*v_pair+1
    u32x4 kr[KP], vr[VP][2];

    auto load_tile = [&](int kt) {
        const int key0 = kt * kPfKTile;
#pragma unroll
        for (int p = 0; p < KP; ++p) {
            int row = key0 + k_row + p * kKRowsPerPass;
            row = row < s ? row : s - 1;
            kr[p] = *(const u32x4 *)(kb + (size_t)row * tok_bytes + k_chunk * 16);
        }
#pragma unroll
        for (int p = 0; p < VP; ++p)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                int row = key0 + 2 * v_pair + u;
                row = row < s ? row : s - 1;
                vr[p][u] = *(const u32x4 *)(vb + (size_t)row * tok_bytes + (v_chunk + 8 * p) * 16);
            }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int p = 0; p < KP; ++p)
            *(u32x4 *)(ks + (k_row + p * kKRowsPerPass) * kKStride + k_chunk * 16) = kr[p];
#pragma unroll
        for (int p = 0; p < VP; ++p) {
            const u32x4 x = vr[p][0], y = vr[p][1];
            const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
            char *dst = vt + ((v_chunk + 8 * p) * 8) * kVStride + v_pair * 4;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                // element 2w of both keys, then element 2w+1 of both keys
                *(uint32_t *)(dst + (2 * w) * kVStride) = (xs[w] & 0xffffu) | (ys[w] << 16);
                *(uint32_t *)(dst + (2 * w + 1) * kVStride) = (xs[w] >> 16) | (ys[w] & 0xffff0000u);
            }
        }
    };

    pf_f32x16 o[ND];
#pragma unroll
    for (int t = 0; t < ND; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
    float m = -INFINITY;  // running maximum of the scaled scores (log2 domain)
    float l = 0.f;        // this lane's share of the running denominator

    load_tile(0);
    for (int kt = 0; kt < nkt; ++kt) {
        __syncthreads();  // every wave is done reading the previous tile
        store_tile();
        __syncthreads();
        if (kt + 1 < nkt) load_tile(kt + 1);  // in flight while this tile is computed
        const int key0 = kt * kPfKTile;
        if (key0 > row0 + 31) continue;  // wave-uniform: the whole tile lies in this wave's future

        // S^T = K Q^T for the two 32-key halves of the tile
        pf_f32x16 sc[2];
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[kh][e] = 0.f;
            const char *krow = ks + (kh * 32 + r) * kKStride + hh * 16;
#pragma unroll
            for (int c = 0; c < NC; ++c) sc[kh] = PfMath<E>::mfma(*(const u32x4 *)(krow + c * 32), qf[c], sc[kh]);
        }
        if (key0 + kPfKTile - 1 > row0) {  // wave-uniform: the tile crosses the diagonal
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + kh * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (key > qrow) sc[kh][e] = -INFINITY;
                }
        }
        float mx = sc[0][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sc[0][e]);
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[1][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx * scale_log2e);  // finite: key 0 is visible to every row
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        l *= alpha;
        uint32_t pb[4][4];  // probabilities of 4 chunks of 16 keys, rounded to the storage type
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[kh][e], scale_log2e, -m_new));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[kh][e + 1], scale_log2e, -m_new));
                l += p0 + p1;
                pb[kh * 2 + (e >> 3)][(e & 7) >> 1] = PfMath<E>::pack2(p0, p1);
            }
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {  // wave-uniform
#pragma unroll
            for (int t = 0; t < ND; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
        }
        // O^T += V^T P^T
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
            const u32x4 pv = u32x4{pb[kc][0], pb[kc][1], pb[kc][2], pb[kc][3]};
#pragma unroll
            for (int t = 0; t < ND; ++t) {
                const char *vrow = vt + (t * 32 + r) * kVStride + (kc * 16 + 4 * hh) * 2;
                const pf_u32x2 a0 = *(const pf_u32x2 *)vrow;
                const pf_u32x2 a1 = *(const pf_u32x2 *)(vrow + 16);
                o[t] = PfMath<E>::mfma(u32x4{a0.x, a0.y, a1.x, a1.y}, pv, o[t]);
            }
        }
    }

    // the denominators of the two half-waves belong to the same rows
    l += __shfl_xor(l, 32, 64);
    if (qrow < s) {
        const float inv = 1.f / l;
        float *ob = out + ((size_t)t0 + qrow) * ((size_t)H * D) + (size_t)h * D;
#pragma unroll
        for (int t = 0; t < ND; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                pf_f32x4 w = {o[t][4 * i] * inv, o[t][4 * i + 1] * inv, o[t][4 * i + 2] * inv, o[t][4 * i + 3] * inv};
                *(pf_f32x4 *)(ob + t * 32 + 8 * i + 4 * hh) = w;
            }
    }
}
