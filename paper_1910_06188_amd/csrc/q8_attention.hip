// FP32 multi-head softmax attention, the operation between the fused Q|K|V FC layer and the
// attention-output FC layer of an encoder layer.  Section 3 keeps Softmax in FP32 and quantizes
// only Embedding and FC layers, so both matrix products around the softmax stay FP32 as well:
//     s[i,j] = scale * <Q[i,:], K[j,:]> (+ mask[j]),   p = softmax_j(s),   ctx[i,:] = sum_j p[i,j] V[j,:]
// Behind it sits the first half of the next FC layer's quantizer (Section 4.1): the abs-max of
// ctx goes to per-workgroup slots, or, with a stored scale (Eq. 4), the int8 codes of ctx are
// written directly (Eq. 1) and ctx itself need not be stored at all.
//
// MFMA kernel (head width 64): a workgroup of four waves owns 128 queries of one (sequence,
// head); each wave keeps its 32 query rows in registers (pre-multiplied by scale * log2 e) and
// walks the keys in stages of 64, K and V tiles staged in LDS and shared by the four waves.
// Scores are formed transposed, S^T = K Q^T, with v_mfma_f32_32x32x2_f32: a lane then holds 16
// keys of ONE query per 32-key block, so the softmax statistics are per-lane loops plus a single
// exchange between the two half-waves, and the probabilities sit exactly where the B operand of
// O^T += V^T P^T wants them -- no data movement between the two products.  Softmax is the
// running-maximum form (scores never exist in memory), evaluated with exp2.
// The key loop is skewed by one stage (the scores of stage i+1 are formed while the softmax of
// stage i runs) and its instruction streams are interleaved by hand, because a wave issues in
// order: see attention_trip.
// Work per (sequence, head): 4 S^2 64 flops; bound by the fp32 matrix pipes (157 TFLOP/s) plus
// the vector arithmetic of the softmax, which on this part is paid on top of the MFMA time
// rather than beside it; the traffic (qkv read once per query block from L2, ctx written once)
// is small beside both.
#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kAtD = 64;                   // head width of the MFMA kernel
constexpr int kAtWaves = 4;                // waves per workgroup
constexpr int kAtThreads = kAtWaves * 64;
constexpr int kAtQW = 32;                  // queries per wave
constexpr int kAtQB = kAtQW * kAtWaves;    // queries per workgroup
constexpr int kAtKB = 64;                  // keys per stage
// LDS row strides in floats.  K rows are read 16 bytes per lane, 16 lanes (keys) per cycle: 68 = 4 (mod 64)
// spreads them over all 64 banks.  V rows are read 4 bytes per lane, the two half-waves four keys apart:
// 4 * 72 = 32 (mod 64) puts the halves on disjoint banks.
constexpr int kAtKStride = 68;
constexpr int kAtVStride = 72;
constexpr int kAtKTile = kAtKB * kAtKStride + kAtKB;     // floats of a K tile in LDS, the stage's mask row behind it
constexpr int kAtVTile = kAtKB * kAtVStride;
constexpr int kAtStageFloats = kAtKTile + kAtVTile;
constexpr int kAtSlots = 2048;             // abs-max slots (= Q8_AMAX_SLOTS)

struct AttnArgs {
    const float* qkv;     // [B*S, 3*heads*d]
    const float* mask;    // [B, S] additive, or null
    float* ctx;           // [B*S, heads*d] or null
    unsigned* slots;      // abs-max slots or null
    const float* q_scale; // stored scale of the next FC or null
    unsigned* q_out;      // int8 codes of ctx, packed four to a dword, or null
    int64_t S;
    int heads;
    int n_qblocks;        // ceil(S / 128)
    int slots_atomic;     // more workgroups than slots: fold with atomics into cleared slots
    float c;              // scale * log2(e)
};

// The score accumulators of a stage start at its mask row (log2 units, -inf beyond the sequence; it sits behind
// the K tile), so the mask costs no addition: s[sub][e] of lane (lq, hi) belongs to key 32 sub + 8 (e/4) + 4 hi + e%4.
__device__ __forceinline__ void attention_load_mask(const float* Ks, int hi, v16f (&s)[2])
{
    const float* mrow = Ks + kAtKB * kAtKStride + 4 * hi;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 mk = *reinterpret_cast<const float4*>(mrow + sub * 32 + 8 * g);
            s[sub][4 * g + 0] = mk.x;
            s[sub][4 * g + 1] = mk.y;
            s[sub][4 * g + 2] = mk.z;
            s[sub][4 * g + 3] = mk.w;
        }
}

// S^T block of one stage (the prologue's; the trips form theirs chunk by chunk): s[sub][e] of lane (lq, hi) =
// mask + <K[32 sub + 8 (e/4) + 4 hi + e%4], c Q[lq]>.  MFMA number 4t + i pairs column 8t + i (lower half-wave)
// with column 8t + 4 + i (upper half-wave) of both operands.
__device__ __forceinline__ void attention_scores(const float* Ks, const float (&q)[32], int lq, int hi, v16f (&s)[2])
{
    attention_load_mask(Ks, hi, s);
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const float4 kf = *reinterpret_cast<const float4*>(Ks + (sub * 32 + lq) * kAtKStride + 4 * hi + 8 * t);
            s[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.x, q[4 * t + 0], s[sub], 0, 0, 0);
            s[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.y, q[4 * t + 1], s[sub], 0, 0, 0);
            s[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.z, q[4 * t + 2], s[sub], 0, 0, 0);
            s[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.w, q[4 * t + 3], s[sub], 0, 0, 0);
        }
}

// Global -> registers -> LDS staging of the K and V tiles (and the mask row) of a stage.  Thread t carries chunks
// t, t + 256, ... of the 64 x 16 float4 chunks of a tile: chunk i is key st_key + 16 i, 16-byte column st_ch.
// Offsets within the sequence fit 32 bits (checked by the launcher); rows beyond the sequence repeat the last one.
struct AttnStager {
    const float *kbase, *vbase;   // K and V of token 0 of this sequence and head (wave-uniform)
    const float* mrow;            // mask row of the sequence, or null
    float *k_tiles, *v_tiles;     // two (K tile + mask row); two V tiles
    unsigned off_st0, off_16, off_stage, off_last;
    int S32, tid, st_key, st_ch;
    float4 k0, k1, k2, k3, v0, v1, v2, v3;
    float m;

    __device__ __forceinline__ unsigned off(int stage, int i) const
    {
        return min(off_st0 + (unsigned)stage * off_stage + (unsigned)i * off_16, off_last);
    }
    __device__ __forceinline__ static float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
    __device__ __forceinline__ void fetch_k01(int stage) { k0 = ld4(kbase + off(stage, 0)); k1 = ld4(kbase + off(stage, 1)); }
    __device__ __forceinline__ void fetch_k23(int stage)
    {
        k2 = ld4(kbase + off(stage, 2));
        k3 = ld4(kbase + off(stage, 3));
        if (mrow) m = mrow[min(stage * kAtKB + (tid & 63), S32 - 1)];
    }
    __device__ __forceinline__ void fetch_v01(int stage) { v0 = ld4(vbase + off(stage, 0)); v1 = ld4(vbase + off(stage, 1)); }
    __device__ __forceinline__ void fetch_v23(int stage) { v2 = ld4(vbase + off(stage, 2)); v3 = ld4(vbase + off(stage, 3)); }
    // the mask row goes in with the K tile, in log2 units; beyond the sequence -inf: weight 0 whatever the
    // (repeated) row holds
    __device__ __forceinline__ float mask_value(int stage) const
    {
        return (stage * kAtKB + tid < S32) ? m * 1.44269504088896341f : -__builtin_inff();
    }
    __device__ __forceinline__ void stash_k(int buf, int stage) const
    {
        float* w = k_tiles + buf * kAtKTile + st_key * kAtKStride + 4 * st_ch;
        *reinterpret_cast<float4*>(w) = k0;
        *reinterpret_cast<float4*>(w + 16 * kAtKStride) = k1;
        *reinterpret_cast<float4*>(w + 32 * kAtKStride) = k2;
        *reinterpret_cast<float4*>(w + 48 * kAtKStride) = k3;
        if (tid < kAtKB) k_tiles[buf * kAtKTile + kAtKB * kAtKStride + tid] = mask_value(stage);
    }
    // One LDS store of the stash that follows trip st: pieces 0-3 the V tile of stage st + 1, 4-7 the K tile
    // of stage nk fetched during that trip, 8 its mask row.
    __device__ __forceinline__ void stash_piece(int j, int st, int nk) const
    {
        if (j < 4) {
            const float4 v = j == 0 ? v0 : j == 1 ? v1 : j == 2 ? v2 : v3;
            *reinterpret_cast<float4*>(v_tiles + ((st + 1) & 1) * kAtVTile + (st_key + 16 * j) * kAtVStride + 4 * st_ch) = v;
        } else if (j < 8) {
            const float4 k = j == 4 ? k0 : j == 5 ? k1 : j == 6 ? k2 : k3;
            *reinterpret_cast<float4*>(k_tiles + (st & 1) * kAtKTile + (st_key + 16 * (j - 4)) * kAtKStride + 4 * st_ch) = k;
        } else if (tid < kAtKB) {
            k_tiles[(st & 1) * kAtKTile + kAtKB * kAtKStride + tid] = mask_value(nk);
        }
    }
    __device__ __forceinline__ void stash_v(int buf) const
    {
        float* w = v_tiles + buf * kAtVTile + st_key * kAtVStride + 4 * st_ch;
        *reinterpret_cast<float4*>(w) = v0;
        *reinterpret_cast<float4*>(w + 16 * kAtVStride) = v1;
        *reinterpret_cast<float4*>(w + 32 * kAtVStride) = v2;
        *reinterpret_cast<float4*>(w + 48 * kAtVStride) = v3;
    }
};

// One trip of the key loop, skewed by a stage: the vector ALU runs the running-maximum softmax of the
// current stage's scores `sc` (log2 units, mask included) while -- kMore -- the matrix pipe forms the next stage's
// scores `sn` from the K tile Kn, its accumulators starting at that stage's mask row; then O^T += V^T P^T of the current stage.  A wave issues in order, so anything
// that waits (an LDS read used at once, a block of address arithmetic and loads, arithmetic behind a run of
// MFMAs) stops its MFMAs as well.  The streams are therefore cut into eight chunks issued in a fixed pattern
// (scheduling groups): every chunk first requests what the NEXT chunk needs from LDS, then alternates one
// MFMA with a few vector instructions.
//   chunks 1-3: row maximum of this lane's 32 scores; exchange between the half-waves
//   chunk  3  : reference maximum m; if it has to move, everything accumulated so far shrinks by 2^(m_old - m)
//   chunks 4-7: p = 2^(s - m) and their sum
//   chunks 0-3: the tile fetches of the stages ahead (V of stage st + 1, K of stage nk), two loads per chunk:
//               issued between MFMAs they cost the matrix pipe nothing, issued in a block they stop it
template <bool kMore>
__device__ __forceinline__ void attention_trip(const float* Kn, const float* Vs, const float (&q)[32], int lq, int hi,
                                               v16f (&sc)[2], v16f (&sn)[2], v16f (&o)[2], float& m_run, float& l_run,
                                               AttnStager& sg, int st, int nk)
{
    float mx = -__builtin_inff(), m_new = 0.0f, psum = 0.0f;
    const float* krow = Kn + lq * kAtKStride + 4 * hi;     // sub-block 1 is 32 rows further on
    float4 kf[2], kf_next[2];
    if (kMore) {
        attention_load_mask(Kn, hi, sn);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) kf[sub] = *reinterpret_cast<const float4*>(krow + sub * 32 * kAtKStride);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        // LDS requests for the next chunk: its K fragments
        if (kMore && t < 7) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
                kf_next[sub] = *reinterpret_cast<const float4*>(krow + sub * 32 * kAtKStride + 8 * (t + 1));
        }
        if (kMore) {
            if (t == 0) sg.fetch_v01(st + 1);
            if (t == 1) sg.fetch_v23(st + 1);
            if (t == 2) sg.fetch_k01(nk);
            if (t == 3) sg.fetch_k23(nk);
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                sn[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[sub].x, q[4 * t + 0], sn[sub], 0, 0, 0);
                sn[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[sub].y, q[4 * t + 1], sn[sub], 0, 0, 0);
                sn[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[sub].z, q[4 * t + 2], sn[sub], 0, 0, 0);
                sn[sub] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[sub].w, q[4 * t + 3], sn[sub], 0, 0, 0);
            }
        }
        if (t >= 1 && t <= 3) {
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int grp = 3 * (t - 1) + j;
                if (grp < 8) {
                    const int sub = grp >> 2, g = grp & 3;   // group = 4 consecutive keys
                    mx = __builtin_fmaxf(mx, __builtin_fmaxf(__builtin_fmaxf(sc[sub][4 * g], sc[sub][4 * g + 1]),
                                                             __builtin_fmaxf(sc[sub][4 * g + 2], sc[sub][4 * g + 3])));
                }
            }
            if (t == 3) {
                // both half-waves hold keys of the same query: swap the halves of two copies and take the maximum.
                // Key 0 of stage 0 is always inside the sequence, so the maximum is finite from the first stage on.
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                const float row_max = __builtin_fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                // The reference maximum moves only when some row of the wave outgrows it by more than 2^8: below
                // that the probabilities are merely up to 256 times larger (harmless in binary32, and the final
                // division takes it out again), and the 32 multiplications that shrink O are saved.  The first
                // stage always moves it (the reference starts at -inf).
                if (__builtin_amdgcn_ballot_w64(row_max > m_run + 8.0f) != 0) {
                    const float m_up = __builtin_fmaxf(m_run, row_max);
                    const float alpha = __builtin_amdgcn_exp2f(m_run - m_up);
                    m_run = m_up;
                    l_run *= alpha;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        o[0][e] *= alpha;
                        o[1][e] *= alpha;
                    }
                }
                m_new = m_run;
            }
        } else if (t >= 4) {
#pragma unroll
            for (int i = 8 * (t - 4); i < 8 * (t - 4) + 8; ++i) {
                sc[i >> 4][i & 15] = __builtin_amdgcn_exp2f(sc[i >> 4][i & 15] - m_new);
                psum += sc[i >> 4][i & 15];
            }
        }
        if (kMore) {   // issue order within the chunk: the LDS reads, then one MFMA, four vector instructions, one MFMA, ...
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x402, 4, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        kf[0] = kf_next[0];
        kf[1] = kf_next[1];
    }
    l_run += psum;
    // O^T += V^T P^T: MFMA pair i = (sub, e) joins key 32 sub + 8 (e/4) + e%4 (lower half-wave) with the key four
    // further on (upper half-wave) -- the keys whose probabilities the two halves hold in register e.  The V
    // operands of a pair are read kAhead pairs before their MFMAs (explicit ring, fenced so that it stays that
    // way), and -- kMore -- the tiles fetched above go to LDS one store at a time under the last pairs (their
    // buffers were last read in the previous trip).
    constexpr int kAhead = 4;
    float va[kAhead + 1][2];
    const float* vcol = Vs + 4 * hi * kAtVStride + lq;
    auto vkey = [](int i) { return (i >> 4) * 32 + 8 * ((i & 15) >> 2) + (i & 3); };
#pragma unroll
    for (int i = 0; i < kAhead; ++i) {
        va[i][0] = vcol[vkey(i) * kAtVStride];
        va[i][1] = vcol[vkey(i) * kAtVStride + 32];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        if (i + kAhead < 32) {
            va[(i + kAhead) % (kAhead + 1)][0] = vcol[vkey(i + kAhead) * kAtVStride];
            va[(i + kAhead) % (kAhead + 1)][1] = vcol[vkey(i + kAhead) * kAtVStride + 32];
        }
        o[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[i % (kAhead + 1)][0], sc[i >> 4][i & 15], o[0], 0, 0, 0);
        o[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[i % (kAhead + 1)][1], sc[i >> 4][i & 15], o[1], 0, 0, 0);
        if (kMore && i >= 20 && i < 29) sg.stash_piece(i - 20, st, nk);
        __builtin_amdgcn_sched_barrier(0);
    }
}

__global__ __launch_bounds__(kAtThreads, 2) void attention_mfma_kernel(AttnArgs a)
{
    extern __shared__ __align__(16) float lds[];   // K tiles (+ mask rows) of two stages, then V tiles of two stages
    __shared__ unsigned wave_amax[kAtWaves];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lq = lane & 31, hi = lane >> 5;
    // Workgroups of one (sequence, head) are neighbours in the logical order; each XCD takes a contiguous
    // run of it so that they find the K and V rows in the same L2.
    int wid = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) wid = (wid & 7) * (total >> 3) + (wid >> 3);
    const int qb = wid % a.n_qblocks;
    const int bh = wid / a.n_qblocks;
    const int h = bh % a.heads;
    const int64_t b = bh / a.heads;
    const int64_t S = a.S, HD = (int64_t)a.heads * kAtD, ld = 3 * HD;
    const float* base = a.qkv + b * S * ld + (int64_t)h * kAtD;   // Q of token 0 of this sequence and head
    const int64_t q0 = (int64_t)qb * kAtQB + wave * kAtQW;

    AttnStager sg;
    const int S32 = (int)S, ld32 = (int)ld;
    const int n_stages = (S32 + kAtKB - 1) / kAtKB;
    sg.S32 = S32;
    sg.tid = tid;
    sg.st_key = tid >> 4;
    sg.st_ch = tid & 15;
    sg.kbase = base + HD;
    sg.vbase = base + 2 * HD;
    sg.mrow = a.mask ? a.mask + b * S : nullptr;
    sg.k_tiles = lds;
    sg.v_tiles = lds + 2 * kAtKTile;
    // offset (in floats, from kbase / vbase) of this thread's chunk 0 of stage 0, the steps to the next chunk and
    // the next stage, and the offset of the same column in the last row of the sequence
    sg.off_st0 = (unsigned)sg.st_key * (unsigned)ld32 + 4u * sg.st_ch;
    sg.off_16 = 16u * (unsigned)ld32;
    sg.off_stage = (unsigned)kAtKB * (unsigned)ld32;
    sg.off_last = (unsigned)(S32 - 1) * (unsigned)ld32 + 4u * sg.st_ch;
    sg.m = 0.0f;
    float* const k_tiles = sg.k_tiles;
    float* const v_tiles = sg.v_tiles;

    v16f o[2];           // O^T: o[blk][e] = ctx[query lq][column 32 blk + 8 (e/4) + 4 hi + e%4], not yet normalised
#pragma unroll
    for (int e = 0; e < 16; ++e) o[0][e] = o[1][e] = 0.0f;
    float m_run = -__builtin_inff();   // running maximum of this lane's query (log2 units), same in both half-waves
    float l_run = 0.0f;                // this lane's share of the running denominator

    // The loop is skewed by one stage: trip st forms the scores of stage st + 1 on the matrix pipe while the
    // vector ALU runs the softmax of stage st, then accumulates P V of stage st.  So K runs one stage ahead
    // of V in LDS, and two ahead in the staging registers.
    v16f s_cur[2], s_nxt[2];
    const int last = n_stages - 1;
    sg.fetch_k01(0);
    sg.fetch_k23(0);
    // The wave's queries, requested behind the first K tile so that the two latencies overlap: lane (lq, hi)
    // holds, for t = 0..7, columns 8t + 4hi .. 8t + 4hi + 3 of query lq, times scale * log2 e.  A row beyond
    // the sequence repeats the last one (computed, never stored).
    float q[32];
    float4 qraw[8];
    {
        const int64_t qrow = (q0 + lq < S) ? q0 + lq : S - 1;
        const float4* qp = reinterpret_cast<const float4*>(base + qrow * ld) + hi;
#pragma unroll
        for (int t = 0; t < 8; ++t) qraw[t] = qp[2 * t];
    }
    sg.stash_k(0, 0);
    sg.fetch_v01(0);
    sg.fetch_v23(0);
    sg.fetch_k01(min(1, last));
    sg.fetch_k23(min(1, last));
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        q[4 * t + 0] = qraw[t].x * a.c;
        q[4 * t + 1] = qraw[t].y * a.c;
        q[4 * t + 2] = qraw[t].z * a.c;
        q[4 * t + 3] = qraw[t].w * a.c;
    }
    __syncthreads();
    attention_scores(k_tiles, q, lq, hi, s_cur);
    sg.stash_v(0);
    sg.stash_k(1, min(1, last));
    __syncthreads();

    for (int st = 0; st < last; ++st) {
        attention_trip<true>(k_tiles + ((st + 1) & 1) * kAtKTile, v_tiles + (st & 1) * kAtVTile, q, lq, hi, s_cur, s_nxt, o, m_run,
                             l_run, sg, st, min(st + 2, last));
        __syncthreads();
        s_cur[0] = s_nxt[0];
        s_cur[1] = s_nxt[1];
    }
    attention_trip<false>(k_tiles, v_tiles + (last & 1) * kAtVTile, q, lq, hi, s_cur, s_nxt, o, m_run, l_run, sg, last, last);

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    const bool live = q0 + lq < S;
    const float qs = a.q_out ? a.q_scale[0] : 0.0f;
    float amax = 0.0f;
    const int64_t out_off = (b * S + q0 + lq) * HD + (int64_t)h * kAtD + 4 * hi;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float4 v;
            v.x = o[blk][4 * g + 0] * inv;
            v.y = o[blk][4 * g + 1] * inv;
            v.z = o[blk][4 * g + 2] * inv;
            v.w = o[blk][4 * g + 3] * inv;
            if (live) {
                const int64_t off = out_off + 32 * blk + 8 * g;
                if (a.ctx) *reinterpret_cast<float4*>(a.ctx + off) = v;
                if (a.q_out)  // Eq. 1 with the stored scale of the next FC layer, four codes per lane
                    a.q_out[off >> 2] = ((unsigned)quantize_code(v.x, qs) & 0xffu) | (((unsigned)quantize_code(v.y, qs) & 0xffu) << 8) |
                                        (((unsigned)quantize_code(v.z, qs) & 0xffu) << 16) | ((unsigned)quantize_code(v.w, qs) << 24);
                amax = __builtin_fmaxf(amax, __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(v.x), __builtin_fabsf(v.y)),
                                                            __builtin_fmaxf(__builtin_fabsf(v.z), __builtin_fabsf(v.w))));
            }
        }
    if (a.slots) {
        unsigned m = wave_max_u32(__float_as_uint(amax));  // non-negative floats order like their bit patterns
        if (lane == 0) wave_amax[wave] = m;
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 1; w < kAtWaves; ++w) m = max(m, wave_amax[w]);
            if (a.slots_atomic) {
                if (m) atomicMax(a.slots + (blockIdx.x % kAtSlots), m);
            } else {
                a.slots[blockIdx.x] = m;
            }
        }
        if (!a.slots_atomic && blockIdx.x == 0)  // slots no workgroup owns
            for (int i = gridDim.x + tid; i < kAtSlots; i += kAtThreads) a.slots[i] = 0u;
    }
}

// Any head width and alignment: one wave per (sequence, head, query).  Scores go to LDS, the softmax is the
// plain three-step form, then each lane sums its columns of V.  Slow; same tolerance.
__global__ __launch_bounds__(64) void attention_generic_kernel(const float* __restrict__ qkv, const float* __restrict__ mask,
                                                               float* __restrict__ ctx, unsigned* __restrict__ slots,
                                                               const float* __restrict__ q_scale, int8_t* __restrict__ q_out,
                                                               int64_t S, int heads, int d, float c)
{
    extern __shared__ __align__(16) float p[];   // S scores / probabilities
    const int lane = threadIdx.x;
    const int64_t i = blockIdx.x % S;
    const int64_t bh = blockIdx.x / S;
    const int h = (int)(bh % heads);
    const int64_t b = bh / heads;
    const int64_t HD = (int64_t)heads * d, ld = 3 * HD;
    const float* qrow = qkv + (b * S + i) * ld + (int64_t)h * d;
    float mx = -__builtin_inff();
    for (int64_t j = lane; j < S; j += 64) {
        const float* krow = qkv + (b * S + j) * ld + HD + (int64_t)h * d;
        float dot = 0.0f;
        for (int k = 0; k < d; ++k) dot = __builtin_fmaf(qrow[k] * c, krow[k], dot);
        if (mask) dot += mask[b * S + j] * 1.44269504088896341f;
        p[j] = dot;
        mx = __builtin_fmaxf(mx, dot);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = __builtin_fmaxf(mx, __shfl_xor(mx, off, 64));
    float den = 0.0f;
    for (int64_t j = lane; j < S; j += 64) {
        const float e = __builtin_amdgcn_exp2f(p[j] - mx);
        p[j] = e;
        den += e;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) den += __shfl_xor(den, off, 64);
    __syncthreads();
    const float inv = 1.0f / den;
    const float qs = q_out ? q_scale[0] : 0.0f;
    float amax = 0.0f;
    for (int k = lane; k < d; k += 64) {
        const float* vcol = qkv + b * S * ld + 2 * HD + (int64_t)h * d + k;
        float acc = 0.0f;
        for (int64_t j = 0; j < S; ++j) acc = __builtin_fmaf(p[j], vcol[j * ld], acc);
        const float v = acc * inv;
        const int64_t off = (b * S + i) * HD + (int64_t)h * d + k;
        if (ctx) ctx[off] = v;
        if (q_out) q_out[off] = (int8_t)quantize_code(v, qs);
        amax = __builtin_fmaxf(amax, __builtin_fabsf(v));
    }
    if (slots) {
        const unsigned m = wave_max_u32(__float_as_uint(amax));
        if (lane == 0 && m) atomicMax(slots + (blockIdx.x % kAtSlots), m);
    }
}

__global__ void attention_slots_clear_kernel(unsigned* slots)
{
    for (int i = threadIdx.x; i < kAtSlots; i += 256) slots[i] = 0u;
}

static bool at_aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int attention_generic_max_s() { return 16384; }   // scores of one query in 64 KiB of LDS

bool attention_mfma_eligible(const float* qkv, int64_t B, int64_t S, int heads, int d, const float* ctx, const int8_t* q_out)
{
    const int64_t wgs = B * heads * ((S + kAtQB - 1) / kAtQB);
    // 32-bit arithmetic inside: the workgroup count, and offsets within one sequence of qkv
    return d == kAtD && at_aligned(qkv, 16) && (!ctx || at_aligned(ctx, 16)) && at_aligned(q_out, 4) &&
           wgs < ((int64_t)1 << 31) && S * 3 * heads * kAtD < ((int64_t)1 << 31);
}

int launch_attention(const float* qkv, int64_t B, int64_t S, int heads, int d, const float* mask, float scale, float* ctx,
                     float* amax_slots, const float* q_scale, int8_t* q_out, hipStream_t st)
{
    unsigned* slots = reinterpret_cast<unsigned*>(amax_slots);
    if (B == 0) {
        if (slots) hipLaunchKernelGGL(attention_slots_clear_kernel, dim3(1), dim3(256), 0, st, slots);
        return hipGetLastError() == hipSuccess ? 0 : 1;
    }
    const float c = scale * 1.44269504088896341f;
    const int64_t n_qblocks = (S + kAtQB - 1) / kAtQB;
    const int64_t wgs = B * heads * n_qblocks;
    if (attention_mfma_eligible(qkv, B, S, heads, d, ctx, q_out)) {
        AttnArgs a;
        a.qkv = qkv;
        a.mask = mask;
        a.ctx = ctx;
        a.slots = slots;
        a.q_scale = q_scale;
        a.q_out = reinterpret_cast<unsigned*>(q_out);
        a.S = S;
        a.heads = heads;
        a.n_qblocks = (int)n_qblocks;
        a.slots_atomic = wgs > kAtSlots;
        a.c = c;
        if (slots && a.slots_atomic) hipLaunchKernelGGL(attention_slots_clear_kernel, dim3(1), dim3(256), 0, st, slots);
        static bool attr_set = false;   // more than 64 KiB of dynamic LDS has to be asked for once
        const size_t lds_bytes = 2 * kAtStageFloats * sizeof(float);
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(attention_mfma_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
                return 1;
            attr_set = true;
        }
        hipLaunchKernelGGL(attention_mfma_kernel, dim3((unsigned)wgs), dim3(kAtThreads), lds_bytes, st, a);
    } else {
        const int64_t blocks = B * heads * S;
        if (blocks >= ((int64_t)1 << 31)) return 1;
        if (slots) hipLaunchKernelGGL(attention_slots_clear_kernel, dim3(1), dim3(256), 0, st, slots);
        hipLaunchKernelGGL(attention_generic_kernel, dim3((unsigned)blocks), dim3(64), (size_t)S * sizeof(float), st, qkv,
                           mask, ctx, slots, q_scale, q_out, S, heads, d, c);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8
