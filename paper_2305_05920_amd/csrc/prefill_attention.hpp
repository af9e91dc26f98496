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
// tiles of 64 tokens, staged once per workgroup in LDS as they lie in memory ([token][d],
// rows padded against bank conflicts).  The key operand is a plain 16-byte LDS read; the
// value operand needs 4 consecutive tokens of one head-dim index per lane, which is what
// the LDS transpose read of gfx950 (ds_read_b64_tr_b16) returns: in a group of 16 lanes,
// lane L receives the 2-byte element L % 4 of the 8 bytes that lanes 4e + L/4 (e = 0..3)
// point at, i.e. column L of a 4 x 16 block whose rows those lanes address.
//
// Per tile a wave computes the transposed score tile S^T = K Q^T (keys x query rows): in
// the accumulator layout of the 32x32 instruction a lane then holds 16 keys of ONE query
// row (row = lane % 32, the other 16 keys sit in lane ^ 32), so the softmax statistics
// are per-lane scalars and need one exchange between the two half-waves.  The same
// registers, rounded to the storage type, are exactly the B operand of O^T = V^T P^T for
// the key order k = 8*(e/4) + 4*(lane/32) + e%4, which the reads of V follow; no
// cross-lane movement of the probabilities is needed.  At the end a wave passes its output
// tile through LDS so that every global store covers whole 256-byte pieces of a row.
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
typedef short pf_i16x4 __attribute__((ext_vector_type(4)));

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
    // acc + lo + hi of a packed pair
    static __device__ __forceinline__ float add_pair(uint32_t pk, float acc) {
        const pf_bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(pf_bf16x2, pk), ones, acc, false);
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
    static __device__ __forceinline__ float add_pair(uint32_t pk, float acc) {
        const pf_f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(pf_f16x2, pk), ones, acc, false);
    }
};

// the value lane (l ^ 32) holds: one cross-half swap on the vector pipe, no LDS round trip
__device__ __forceinline__ float pf_other_half(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (uint32_t)(threadIdx.x & 32 ? sw[0] : sw[1]));
}

// One work-list entry: 128 query rows of 8 heads' worth of workgroups.
struct PfItem {
    int32_t t0;        // first token of the job in the packed arrays
    int32_t s;         // prompt length
    int32_t qt_group;  // query tile | head group << 16 (heads 8*group .. 8*group+7)
    int32_t job;       // index of the job in this launch
};
constexpr int kPfMaxItems = 262144;  // entries the pool's work list holds

// Builds the work list of a launch (one workgroup).  offs[J+1], J <= 1024; G head groups; prompts
// of at most 65535 query tiles.
// items[0].t0 receives the entry count, entries follow from items[1].  A job whose offsets
// decrease or leave [0, total_tokens] raises the flag and gets no entry.
__global__ __launch_bounds__(kThreads) void fs_prefill_plan_kernel(const int32_t *__restrict__ offs, int32_t J,
                                                                   int32_t G, long long total_tokens,
                                                                   PfItem *__restrict__ items,
                                                                   int32_t *__restrict__ err)
{
    __shared__ int32_t s_len[kMaxJobsPerLaunch];
    __shared__ int32_t s_t0[kMaxJobsPerLaunch];
    __shared__ uint16_t s_ord[kMaxJobsPerLaunch];   // job by rank, longest prompt first
    __shared__ int32_t s_base[kMaxJobsPerLaunch + 1];  // first entry of the job of that rank
    bool bad = false;
    for (int j = threadIdx.x; j < J; j += kThreads) {
        const long long a = offs[j], b = offs[j + 1];
        const bool ok = a >= 0 && b >= a && b <= total_tokens;
        bad |= !ok;
        s_len[j] = ok ? (int32_t)(b - a) : 0;
        s_t0[j] = (int32_t)a;
    }
    if (bad) atomicOr(err, kErrBadLen);
    __syncthreads();
    for (int j = threadIdx.x; j < J; j += kThreads) {
        const int mine = s_len[j];
        int rank = 0;
        for (int i = 0; i < J; ++i) {
            const int li = s_len[i];
            rank += (li > mine || (li == mine && i < j)) ? 1 : 0;
        }
        s_ord[rank] = (uint16_t)j;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long acc = 0;
        for (int rk = 0; rk < J; ++rk) {
            s_base[rk] = (int32_t)acc;
            acc += (long long)((s_len[s_ord[rk]] + kPfQTile - 1) / kPfQTile) * G;
            if (acc > kPfMaxItems) {  // more work than the list holds: serve what fits, say so
                atomicOr(err, kErrBadLen);
                acc = s_base[rk];
                for (int r2 = rk; r2 <= J; ++r2) s_base[r2] = (int32_t)acc;
                break;
            }
        }
        s_base[J] = (int32_t)acc;
        items[0].t0 = (int32_t)acc;
    }
    __syncthreads();
    const int total = s_base[J];
    for (int e = threadIdx.x; e < total; e += kThreads) {
        int lo = 0, hi = J;  // largest rank with s_base[rank] <= e (ranks without entries share a base)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_base[mid] <= e) lo = mid; else hi = mid;
        }
        const int j = s_ord[lo];
        const int tiles = (s_len[j] + kPfQTile - 1) / kPfQTile;
        const int rem = e - s_base[lo];
        PfItem it;
        it.t0 = s_t0[j];
        it.s = s_len[j];
        it.qt_group = (tiles - 1 - rem % tiles) | ((rem / tiles) << 16);
        it.job = j;
        items[1 + e] = it;
    }
}

// q, k, v: [total_tokens][H][D] (2-byte elements), jobs packed back to back.
// out: [total_tokens][H][D] fp32.  `items` is the work list fs_prefill_plan_kernel wrote: entry
// seq names a job (its first token and length), a group of 8 heads and a query tile.
// Workgroup b runs on die b % 8 as that die's (b / 8)-th workgroup and serves entry b / 8 with
// head 8 * group + b % 8.  The list walks the jobs from the longest down and, inside a
// (job, head group), the query tiles from the last (most keys) to the first: the tiles of a
// (job, head) so run at the same time on one die and find its keys and values in that
// die's L2, and the long items start first.
//
// kWrite: the call is the whole initialization phase of its jobs and also fills their cache
// blocks: token t of job j goes to slot t % 16 of block table[j][t / 16].  The workgroup whose
// query rows ARE the tokens of a key tile (query tile kt / 2) writes that tile while it has it
// staged: keys from LDS with 16 lanes over the 16 slots of a block, so that a wave writes 1 KiB
// of the pool's [d/8][slot][8] key order in one piece, values from the staging registers row by row.
template <typename E, int D, bool kWrite>
__global__ __launch_bounds__(kThreads, 2) void fs_prefill_attn_kernel(
    const char *__restrict__ q, const char *__restrict__ k, const char *__restrict__ v,
    const PfItem *__restrict__ items, float *__restrict__ out, int32_t H, float scale_log2e,
    char *__restrict__ pool, const int32_t *__restrict__ table, int32_t table_stride, int32_t num_blocks,
    int32_t *__restrict__ err)
{
    constexpr int kKStride = D * 2 + 16;  // bytes per staged key row: 16 rows hit 16 different bank groups
    constexpr int kVStride = D * 2 + 32;  // bytes per staged value row: 4 rows of a transpose read do
    constexpr int NC = D / 16;            // 16-wide chunks of the head dimension
    constexpr int ND = D / 32;            // 32-wide tiles of the output's head dimension
    constexpr int kChunks = D / 8;        // 16-byte chunks per token row
    constexpr int kRowsPerPass = kThreads / kChunks;
    constexpr int SP = kPfKTile / kRowsPerPass;  // staging passes per tile
    constexpr int kKBytes = kPfKTile * kKStride;
    constexpr int kVBytes = kPfKTile * kVStride;
    constexpr int kOutCols = D / 2;                   // output columns a wave stages per pass
    constexpr int kOutStride = kOutCols * 4 + 16;     // bytes per staged output row
    static_assert(kWavesPerWg * 32 * kOutStride <= kKBytes + kVBytes, "output staging must fit the tile buffers");
    __shared__ __attribute__((aligned(16))) char lds[kKBytes + kVBytes];
    char *const ks = lds;
    char *const vs = lds + kKBytes;

    const int seq = blockIdx.x / kXcds;
    if (seq >= items[0].t0) return;
    const PfItem item = items[1 + seq];
    const int h = (item.qt_group >> 16) * kXcds + blockIdx.x % kXcds;
    if (h >= H) return;
    const long long t0 = item.t0;
    const int s = item.s, qt = item.qt_group & 0xffff;

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

    // staging role of this thread: 16 bytes of token row st_row (+ kRowsPerPass per pass)
    const int st_row = threadIdx.x / kChunks, st_chunk = threadIdx.x % kChunks;
    u32x4 kr[SP], vr[SP];

    // this thread's byte offset from a tile's first row, per pass (a tile's rows lie
    // tok_bytes apart; 64 rows of at most 16 MB fit 32 bits)
    uint32_t st_off[SP];
#pragma unroll
    for (int p = 0; p < SP; ++p) st_off[p] = (uint32_t)((size_t)(st_row + p * kRowsPerPass) * tok_bytes) + st_chunk * 16;
    auto load_tile = [&](int kt) {
        const size_t tile = (size_t)kt * kPfKTile * tok_bytes;  // wave-uniform
        if (kt * kPfKTile + kPfKTile <= s) {  // the whole tile lies inside the prompt: no address arithmetic per lane
#pragma unroll
            for (int p = 0; p < SP; ++p) {
                kr[p] = *(const u32x4 *)(kb + tile + st_off[p]);
                vr[p] = *(const u32x4 *)(vb + tile + st_off[p]);
            }
        } else {  // the prompt's last tile: rows past its end repeat its last row
#pragma unroll
            for (int p = 0; p < SP; ++p) {
                int row = kt * kPfKTile + st_row + p * kRowsPerPass;
                row = row < s ? row : s - 1;
                kr[p] = *(const u32x4 *)(kb + (size_t)row * tok_bytes + st_chunk * 16);
                vr[p] = *(const u32x4 *)(vb + (size_t)row * tok_bytes + st_chunk * 16);
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int p = 0; p < SP; ++p) {
            *(u32x4 *)(ks + (st_row + p * kRowsPerPass) * kKStride + st_chunk * 16) = kr[p];
            *(u32x4 *)(vs + (st_row + p * kRowsPerPass) * kVStride + st_chunk * 16) = vr[p];
        }
    };

    // A operand number i of O^T += V^T P^T: head-dim rows 32*(i%ND) + r, keys 16*(i/ND) +
    // {4hh..4hh+3, 8+4hh..8+4hh+3} of the staged tile.  In its group of 16 lanes this lane
    // addresses token 4hh + (lane%16)/4 and the 4 head-dim indices 16*((lane/16)%2) + 4*(lane%4) ..
    const char *const vlane = vs + (4 * hh + ((lane & 15) >> 2)) * kVStride + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    auto v_operand = [&](int i) {
        typedef pf_i16x4 __attribute__((address_space(3))) * lds_i16x4_ptr;
        const char *p0 = vlane + (16 * (i / ND)) * kVStride + (i % ND) * 64;
        const pf_i16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)p0);
        const pf_i16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p0 + 8 * kVStride));
        const pf_u32x2 w0 = __builtin_bit_cast(pf_u32x2, a0), w1 = __builtin_bit_cast(pf_u32x2, a1);
        return u32x4{w0.x, w0.y, w1.x, w1.y};
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
        const int key0 = kt * kPfKTile;
        if (kWrite && (kt >> 1) == qt) {  // workgroup-uniform: this tile's tokens are this workgroup's rows
            static_assert(kPfKTile % kBlockTokens == 0 && kPfQTile == 2 * kPfKTile, "tile shapes");
            const size_t chunk = (size_t)kBlockTokens * D * 2;  // bytes of one head's keys (or values) in a block
            const int32_t *trow = table + (size_t)item.job * table_stride;
            // values: this thread's staging registers hold 16 bytes of row st_row (+ kRowsPerPass per pass)
#pragma unroll
            for (int p = 0; p < SP; ++p) {
                const int pos = key0 + st_row + p * kRowsPerPass;
                if (pos < s) {
                    const int bid = pos / kBlockTokens < table_stride ? trow[pos / kBlockTokens] : -1;
                    if ((uint32_t)bid < (uint32_t)num_blocks)
                        *(u32x4 *)(pool + (size_t)bid * (2 * (size_t)H * chunk) + ((size_t)H + h) * chunk +
                                   (size_t)(pos % kBlockTokens) * (D * 2) + st_chunk * 16) = vr[p];
                    else if (st_chunk == 0 && h == 0) atomicOr(err, kErrBadBlock);
                }
            }
            // keys: lane -> slot, so that 16 lanes fill the 256 contiguous bytes of one d/8 chunk
            const int w_slot = threadIdx.x % kBlockTokens, w_rest = threadIdx.x / kBlockTokens;
            constexpr int kPieces = kPfKTile * kChunks / kThreads;  // 16-byte pieces per thread
#pragma unroll
            for (int p = 0; p < kPieces; ++p) {
                const int piece = w_rest + p * (kThreads / kBlockTokens);  // (block in tile, chunk)
                const int blk = piece / kChunks, ch = piece % kChunks;
                const int pos = key0 + blk * kBlockTokens + w_slot;
                if (pos < s) {
                    const int bid = pos / kBlockTokens < table_stride ? trow[pos / kBlockTokens] : -1;
                    if ((uint32_t)bid < (uint32_t)num_blocks)
                        *(u32x4 *)(pool + (size_t)bid * (2 * (size_t)H * chunk) + (size_t)h * chunk +
                                   ((size_t)ch * kBlockTokens + w_slot) * 16) =
                            *(const u32x4 *)(ks + (blk * kBlockTokens + w_slot) * kKStride + ch * 16);
                }
            }
        }
        if (kt + 1 < nkt) load_tile(kt + 1);  // in flight while this tile is computed
        // wave-uniform: the whole tile lies in this wave's future, or the wave has no row of the prompt
        if (key0 > row0 + 31 || row0 >= s) continue;

        // S^T = K Q^T for the two 32-key halves of the tile.  The LDS reads run ahead of the
        // matrix instructions that use them: the operands of a half are in flight while the
        // previous half multiplies, and the first value operands while the second half does.
        pf_f32x16 sc[2];
#pragma unroll
        for (int e = 0; e < 16; ++e) sc[0][e] = 0.f, sc[1][e] = 0.f;
        u32x4 a[NC];
        {
            const char *krow = ks + r * kKStride + hh * 16;
#pragma unroll
            for (int c = 0; c < NC; ++c) a[c] = *(const u32x4 *)(krow + c * 32);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                sc[0] = PfMath<E>::mfma(a[c], qf[c], sc[0]);
                a[c] = *(const u32x4 *)(krow + 32 * kKStride + c * 32);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                sc[1] = PfMath<E>::mfma(a[c], qf[c], sc[1]);
                a[c] = v_operand(c);
            }
            __builtin_amdgcn_sched_barrier(0);
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
        mx = fmaxf(mx, pf_other_half(mx));
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
                const uint32_t pk = PfMath<E>::pack2(p0, p1);
                l = PfMath<E>::add_pair(pk, l);  // the denominator sums what the matrix cores will multiply
                pb[kh * 2 + (e >> 3)][(e & 7) >> 1] = pk;
            }
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {  // wave-uniform
#pragma unroll
            for (int t = 0; t < ND; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
        }
        // O^T += V^T P^T: operand i covers keys 16*(i/ND).. of the tile and output rows
        // 32*(i%ND)..; the first NC operands are already in registers
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4 * ND; ++i) {
            const int kc = i / ND;
            const u32x4 pv = u32x4{pb[kc][0], pb[kc][1], pb[kc][2], pb[kc][3]};
            o[i % ND] = PfMath<E>::mfma(a[i % NC], pv, o[i % ND]);
            if (i + NC < 4 * ND) a[i % NC] = v_operand(i + NC);
            __builtin_amdgcn_sched_barrier(0);  // keep each refill right behind the instruction that frees its registers
        }
    }

    // the denominators of the two half-waves belong to the same rows
    l += pf_other_half(l);
    const float inv = 1.f / l;
    // Output: the wave's 32 x D tile goes through LDS in two passes of D/2 columns, so that a
    // row's columns leave in one piece (16 lanes x 16 bytes) instead of 16 bytes per lane.
    __syncthreads();  // the tile buffers are free
    char *const stage = lds + wave * (32 * kOutStride);
    constexpr int kLanesPerRow = kOutCols / 4;        // lanes that cover a staged row with 16 bytes each
    constexpr int kRowsPerStore = 64 / kLanesPerRow;  // rows one store instruction covers
    const int out_row = lane / kLanesPerRow, out_col = (lane % kLanesPerRow) * 4;
    float *const ob = out + ((size_t)t0 + row0) * ((size_t)H * D) + (size_t)h * D;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int tt = 0; tt < ND / 2; ++tt) {
            const int t = pass * (ND / 2) + tt;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                pf_f32x4 w = {o[t][4 * i] * inv, o[t][4 * i + 1] * inv, o[t][4 * i + 2] * inv, o[t][4 * i + 3] * inv};
                *(pf_f32x4 *)(stage + r * kOutStride + (tt * 32 + 8 * i + 4 * hh) * 4) = w;
            }
        }
        wave_lds_sync();
#pragma unroll
        for (int it = 0; it < 32 / kRowsPerStore; ++it) {
            const int row = it * kRowsPerStore + out_row;
            const pf_f32x4 w = *(const pf_f32x4 *)(stage + row * kOutStride + out_col * 4);
            if (row0 + row < s) *(pf_f32x4 *)(ob + (size_t)row * ((size_t)H * D) + pass * kOutCols + out_col) = w;
        }
        wave_lds_sync();
    }
}
