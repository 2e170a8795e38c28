// i8 MFMA GEMM kernel template of the quantized FC layer (Section 3), gfx950.  Included by
// one translation unit per tile shape (q8_gemm_tile*.hip) so the shapes compile in parallel.
#pragma once
#include <type_traits>

#include "q8_device.h"
#include "q8_epilogue.h"
#include "q8_launch.h"

namespace q8 {

constexpr int kBK = 128;  // bytes (= int8 elements) of K per LDS row and per pipeline stage: one full
                          // 128-byte cache line of every operand row, so no line is fetched twice
constexpr int kKS = kBK / 32;  // 32-byte MFMA k-steps per stage

// LDS rows are kBK = 128 bytes (8 chunks of 16 B).  Chunk c of row r is kept at slot
// c ^ ((r ^ (r >> 3)) & 7): the 16 rows a ds_read_b128 serves per cycle then cover all 64
// banks (measured conflict-free on gfx950; r & 7 alone leaves a 2-way conflict).
__device__ __forceinline__ int swizzle_of_row(int r) { return (r ^ (r >> 3)) & 7; }

// s_waitcnt immediates for gfx9: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8.
__host__ __device__ constexpr int waitcnt_vm(int vm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | (15 << 8); }
__host__ __device__ constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4); }

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of
// tile ids so that the tiles sharing operand rows meet in the same L2.
__device__ __forceinline__ int xcd_remap(int b, int g)
{
    int per = g >> 3, rem = g & 7;
    int xcd = b & 7, idx = b >> 3;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

typedef __attribute__((address_space(3))) char* lds_ptr_t;

// Raw buffer descriptor (gfx9 layout): 48-bit base, stride 0, num_records in bytes.
__device__ __forceinline__ v4i make_rsrc(const void* base, unsigned bytes)
{
    const unsigned long long p = reinterpret_cast<unsigned long long>(base);
    v4i r;
    r[0] = (int)(unsigned)(p & 0xffffffffu);
    r[1] = (int)(unsigned)((p >> 32) & 0xffffu);
    r[2] = (int)bytes;
    r[3] = 0x00020000;
    return r;
}

// 16 bytes per lane from a buffer straight into LDS: lane l lands at M0 + OFF + 16*l and
// reads global byte voff + soff + OFF (the instruction's immediate offset applies to both
// sides).  rsrc, soff and the LDS address are wave-uniform.  Written as asm so that the
// compiler does not pair every later LDS read with a full vmcnt(0) wait; the kernel orders
// these loads against its LDS reads itself (s_waitcnt vmcnt + barrier).
// lds_dma16_first also points M0 at the LDS block (one wait state before the load);
// lds_dma16_next reuses M0, so a run of four 1 KiB blocks costs one M0 write: with a single
// wave per SIMD every instruction issued between two MFMAs counts.
__device__ __forceinline__ void lds_dma16_first(v4i rsrc, unsigned voff, unsigned soff, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_dma16_next(v4i rsrc, unsigned voff, unsigned soff)
{
    static_assert(OFF > 0 && OFF < 4096, "12-bit immediate");
    asm volatile("buffer_load_dwordx4 %0, %1, %2 offen offset:%3 lds" : : "v"(voff), "s"(rsrc), "s"(soff), "n"(OFF) : "memory");
}
// i-th 1 KiB block of a run that starts at lds_run: blocks 4g..4g+3 share one M0 value.
template <int I>
__device__ __forceinline__ void lds_dma16_run(v4i rsrc, unsigned voff, unsigned soff, unsigned lds_run)
{
    if constexpr (I % 4 == 0)
        lds_dma16_first(rsrc, voff, soff, lds_run + I * 1024);
    else
        lds_dma16_next<(I % 4) * 1024>(rsrc, voff - (I % 4) * 1024, soff);
}

// Compile-time loop: the body sees its index as a constant, so accumulator registers
// are always addressed statically.
template <int I, int E, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, E>(f);
    }
}

// Waves per SIMD the kernel is compiled for: a tile whose rings take at most half of the LDS is
// meant to run as two workgroups per compute unit (one's epilogue under the other's main loop),
// which only happens if each wave also stays within half of the register file.
constexpr int mfma_waves_per_simd(int BM, int BN, int SB, int NW)
{
    return ((2 * BM + SB * BN) * kBK <= 80 * 1024 ? 2 : 1) * (NW / 4);
}

// Software-pipelined MFMA kernel.
//
// K is walked in stages of kBK = 128 bytes, four 32-byte k-steps each.  The x tile (A) and
// the w tile (B) each have their own ring of stage buffers in LDS: SA slots for A, SB for B.
//
//   k-steps 0..2 of stage t : ds_read fragments of the next k-step, and -- with SB = 3 -- the
//                             B loads of stage t+3 into the B slot stage t-... left free at the
//                             previous barrier                               || MFMAs
//   wait: own reads of stage t done, own loads of stage t+1 landed;  barrier
//   k-step 3 of stage t     : A loads of stage t+SA into the A slot of stage t (and, with
//                             SB = 2, the B loads of stage t+2 likewise),
//                             ds_read fragments (t+1, k-step 0)              || MFMAs
//
// Why two ring depths: a wave that issues a global->LDS load is held until the texture
// path accepts it (one 1 KiB wave load per ~64 cycles per wave when all four waves load),
// and with one wave per SIMD nothing else feeds the matrix pipe meanwhile.  Measured: more
// than one load per two MFMAs stalls the pipe.  A third B slot lets the B loads spread over
// the first three k-steps, leaving only the A loads for the last one; where LDS cannot hold
// it (SB = 2) all loads fall in the last k-step.
//
// Every memory operation of a k-step is placed by hand behind a given MFMA (LDS reads early,
// global loads at least two MFMAs apart).  Loads past the end of K go through an empty
// buffer descriptor (num_records = 0): the hardware drops them and returns zeros, so the
// vmcnt bookkeeping is the same in every trip and no memory is touched.
//
// kEpi fixes the epilogue at compile time: 0..5 = that exact combination of Q8_EPI_GELU (1),
// Q8_EPI_ABSMAX (2) and Q8_EPI_REQUANT (4) with no accumulator dump; 8 = no flags, residual
// added; -1 = decide at run time (any flags, optional dump, optional residual).  With one wave per SIMD a per-element run-time branch costs
// more than the arithmetic it guards, so the combinations that matter get their own kernel.
template <int BM, int BN, int WGM, int WGN, int SB, int kEpi>
__global__ __launch_bounds__(WGM* WGN * 64, mfma_waves_per_simd(BM, BN, SB, WGM* WGN)) void gemm_mfma_kernel(const int8_t* __restrict__ X,
                                                                   const int8_t* __restrict__ W, int M, int N, int K,
                                                                   int tiles_n, int group_m, Epilogue ep)
{
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    constexpr int SA = 2;
    constexpr bool kGen = kEpi < 0, kPlain = kEpi == 0;
    const bool do_gelu = kGen ? (ep.flags & 1u) != 0 : (kEpi & 1) != 0;
    const bool do_amax = kGen ? (ep.flags & 2u) != 0 : (kEpi & 2) != 0;
    const bool do_req = kGen ? (ep.flags & 4u) != 0 : (kEpi & 4) != 0;
    const bool do_dump = kGen && ep.acc_out != nullptr;
    const bool do_res = kGen ? ep.residual != nullptr : kEpi == 8;
    constexpr int NW = WGM * WGN;
    constexpr int TM = BM / WGM, TN = BN / WGN;  // wave tile
    constexpr int FM = TM / 32, FN = TN / 32;    // 32x32 MFMA blocks per wave tile
    constexpr int A_BYTES = BM * kBK, B_BYTES = BN * kBK;
    constexpr int B_RING = SA * A_BYTES;                         // LDS offset of the B ring
    constexpr int LDS_BYTES = SA * A_BYTES + SB * B_BYTES;
    constexpr int A_LOADS = BM / 8 / NW, B_LOADS = BN / 8 / NW;  // 1 KiB wave loads per stage
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split over the waves");
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert(SB == 2 || SB == 3, "B ring depth");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS is 160 KiB per compute unit");
    static_assert(A_LOADS + B_LOADS <= 63, "vmcnt is a 6-bit counter");

    __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds_base = (unsigned)(size_t)(lds_ptr_t)lds;

    // tile id -> (tm, tn): panels of group_m tile rows, column-major inside a panel
    int pid = xcd_remap(blockIdx.x, gridDim.x);
    const int tiles_m = gridDim.x / tiles_n;
    {
        int panel = pid / (group_m * tiles_n);
        int first = panel * group_m;
        int rows = min(group_m, tiles_m - first);
        int in_panel = pid - panel * group_m * tiles_n;
        pid = (first + in_panel % rows) * tiles_n + in_panel / rows;
    }
    const int m0 = (pid / tiles_n) * BM;
    const int n0 = (pid % tiles_n) * BN;

    // Operand descriptors start at the tile's first row, so the 32-bit offsets only span one tile
    // (at most 256 rows x K bytes) however large the matrices are.
    const int rows_a = min(BM, M - m0), rows_b = min(BN, N - n0);
    const unsigned bytes_a = (unsigned)rows_a * (unsigned)K, bytes_b = (unsigned)rows_b * (unsigned)K;
    const int8_t* Xt = X + (int64_t)m0 * K;
    const int8_t* Wt = W + (int64_t)n0 * K;

    // Per-lane global byte offsets of this lane's chunk in each wave load (k = 0).  One
    // wave load covers 8 rows x 128 B; lane l fills row l/8, slot l%8 of the LDS side.
    // Rows beyond the matrix edge re-read the last row; their products are never stored.
    unsigned a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        int r = (wave * A_LOADS + i) * 8 + (lane >> 3);
        int c = (lane & 7) ^ swizzle_of_row(r);
        a_off[i] = (unsigned)min(r, rows_a - 1) * (unsigned)K + (unsigned)(c * 16);
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        int r = (wave * B_LOADS + i) * 8 + (lane >> 3);
        int c = (lane & 7) ^ swizzle_of_row(r);
        b_off[i] = (unsigned)min(r, rows_b - 1) * (unsigned)K + (unsigned)(c * 16);
    }

    const int KT = K / kBK;
    // Descriptor, k offset and LDS run of this wave's share of one operand tile of stage kt.
    struct Src {
        v4i rsrc;
        unsigned koff, dst;
    };
    auto src_a = [&](int kt, int slot) {
        const bool live = kt < KT;  // past the end of K: empty descriptor, nothing is fetched
        return Src{make_rsrc(Xt, live ? bytes_a : 0u), live ? (unsigned)(kt * kBK) : 0u,
                   lds_base + (unsigned)(slot * A_BYTES + wave * A_LOADS * 1024)};
    };
    auto src_b = [&](int kt, int slot) {
        const bool live = kt < KT;
        return Src{make_rsrc(Wt, live ? bytes_b : 0u), live ? (unsigned)(kt * kBK) : 0u,
                   lds_base + (unsigned)(B_RING + slot * B_BYTES + wave * B_LOADS * 1024)};
    };
    auto load_all_a = [&](const Src& q) {
        static_for<0, A_LOADS>([&](auto ic) { lds_dma16_run<decltype(ic)::value>(q.rsrc, a_off[decltype(ic)::value], q.koff, q.dst); });
    };
    auto load_all_b = [&](const Src& q) {
        static_for<0, B_LOADS>([&](auto ic) { lds_dma16_run<decltype(ic)::value>(q.rsrc, b_off[decltype(ic)::value], q.koff, q.dst); });
    };

    // Fragment addressing: lane l of a 32x32x32 MFMA supplies row (l % 32) and the
    // 16 k-bytes numbered (l / 32) of a 32-byte k-step, for both operands.
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, hi = lane >> 5;
    int a_frag_off[FM][kKS], b_frag_off[FN][kKS];  // [block][k-step] byte offset inside a stage slot
#pragma unroll
    for (int f = 0; f < FM; ++f) {
        int r = wm * TM + f * 32 + l32;
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) a_frag_off[f][ks] = r * kBK + (((ks * 2 + hi) ^ swizzle_of_row(r)) << 4);
    }
#pragma unroll
    for (int f = 0; f < FN; ++f) {
        int r = wn * TN + f * 32 + l32;
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks)
            b_frag_off[f][ks] = B_RING + r * kBK + (((ks * 2 + hi) ^ swizzle_of_row(r)) << 4);
    }

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    v4i fa[2][FM], fb[2][FN];  // fragments of the current / next k-step, double buffered in registers

    // The epilogue's per-column inputs (activation scale, weight scale of the column's group, bias)
    // are fetched now and only used after the main loop: fetched there, their latency would sit
    // between the last MFMA and the first store of every tile.
    const float sx = ep.sx[0];
    float sw_col[FN], bias_col[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = min(n0 + wn * TN + j * 32 + l32, N - 1);
        sw_col[j] = ep.sw[n / ep.cols_per_group];
        bias_col[j] = ep.bias ? ep.bias[n] : 0.0f;
    }

    // The descriptors of the epilogue start at the tile's first row, so byte offsets stay below BM * N * 4
    // whatever the size of y (N * BM * 4 < 2^31 is all that is asked of the shape).
    const bool interior = (m0 + BM <= M) && (n0 + BN <= N) && ((int64_t)N * BM * 4 < ((int64_t)1 << 31));
    const int64_t tile_row0 = (int64_t)m0 * N;
    const int row0 = wm * TM + 4 * hi;  // first row this lane stores, counted from the tile's first row

    // Residual of an interior tile: per 32x32 block 16 loads per lane, each the 2 x 128 contiguous bytes
    // its store will cover, kept kResAhead blocks ahead of the block being dequantized and stored.  The
    // first blocks are fetched here, ahead of the main loop, so that no store of the epilogue waits for
    // a fetch from memory (fetched there, 16 KB in flight per workgroup and the memory latency bound the
    // whole tile).  They are older than every operand load, so the loop's own counted waits cover them.
    // y may be the residual tensor itself: every element is read and written by the same lane, the read first.
    // (The run-time-flag kernel has no registers to spare: it stays one block ahead and starts after the loop.)
    constexpr int kResAhead = kGen ? 1 : 2, kResSlots = kResAhead + 1;
    const bool fetch_res = do_res && interior;
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(fetch_res ? ep.residual + tile_row0 : ep.residual), 0, fetch_res ? BM * N * 4 : 0, 0x00020000);
    float res[kResSlots][16];
    auto fetch_residual = [&](auto bc) {
        constexpr int b = decltype(bc)::value, j = b / FM, i = b % FM;
        const int elem0 = row0 * N + n0 + wn * TN + j * 32 + l32;
        static_for<0, 16>([&](auto ec) {
            constexpr int e = decltype(ec)::value;
            constexpr int dm = i * 32 + 8 * (e >> 2) + (e & 3);
            res[b % kResSlots][e] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rres, elem0 * 4, dm * N * 4, 0));
        });
    };
    auto fetch_first_residuals = [&]() {
        if (fetch_res) static_for<0, (kResAhead < FM * FN ? kResAhead : FM * FN)>([&](auto bc) { fetch_residual(bc); });
    };
    if constexpr (!kGen) fetch_first_residuals();

    // Prologue: stages 0 and 1 of both operands; wait for stage 0.
    load_all_a(src_a(0, 0));
    load_all_b(src_b(0, 0));
    load_all_a(src_a(1, 1));
    load_all_b(src_b(1, 1));
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(A_LOADS + B_LOADS));
    __syncthreads();
#pragma unroll
    for (int f = 0; f < FM; ++f) fa[0][f] = *reinterpret_cast<const v4i*>(lds + a_frag_off[f][0]);
#pragma unroll
    for (int f = 0; f < FN; ++f) fb[0][f] = *reinterpret_cast<const v4i*>(lds + b_frag_off[f][0]);

    constexpr int NM = FM * FN, NR = FM + FN;
    int a_slot = 0, b_slot = 0;  // ring slots of the stage being consumed
    for (int kt = 0; kt < KT; ++kt) {
        const int a_next = a_slot ^ 1;
        const int b_next = (b_slot + 1 == SB) ? 0 : b_slot + 1;
        const int b_prev = (b_slot == 0) ? SB - 1 : b_slot - 1;
        const char* cur_a = lds + a_slot * A_BYTES;
        const char* cur_b = lds + b_slot * B_BYTES;
        // SB = 3: the B slot of stage kt-1 was left by every wave at the last barrier (at
        // kt = 0 it has not been used yet); it takes the B tile of stage kt+2
        const Src qb3 = src_b(kt + 2, b_prev);
        // k-steps 0..2
        static_for<0, kKS - 1>([&](auto ksc) {
            constexpr int ks = decltype(ksc)::value;
            constexpr int C = ks & 1, Nx = (ks + 1) & 1;
            constexpr int bl0 = (SB == 3) ? (B_LOADS * ks) / (kKS - 1) : 0;
            constexpr int bl1 = (SB == 3) ? (B_LOADS * (ks + 1)) / (kKS - 1) : 0;
            constexpr int ND = bl1 - bl0;
            static_for<0, NM>([&](auto ic) {
                constexpr int idx = decltype(ic)::value;
                constexpr int i = idx / FN, j = idx % FN;
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[C][i], fb[C][j], acc[i][j], 0, 0, 0);
                // fragments of k-step ks+1: two reads behind each of the first MFMAs
                static_for<2 * idx, (2 * idx + 2 < NR ? 2 * idx + 2 : NR)>([&](auto rc) {
                    constexpr int r = decltype(rc)::value;
                    if constexpr (r < FM)
                        fa[Nx][r] = *reinterpret_cast<const v4i*>(cur_a + a_frag_off[r][ks + 1]);
                    else
                        fb[Nx][r - FM] = *reinterpret_cast<const v4i*>(cur_b + b_frag_off[r - FM][ks + 1]);
                });
                // B loads, spread over the k-step
                static_for<(ND * idx) / NM, (ND * (idx + 1)) / NM>([&](auto lc) {
                    constexpr int l = bl0 + decltype(lc)::value;
                    lds_dma16_run<l>(qb3.rsrc, b_off[l], qb3.koff, qb3.dst);
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        // own LDS reads of stage kt are complete and own loads of stage kt+1 have landed;
        // with SB = 3 the B loads just issued may still be in flight
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(SB == 3 ? B_LOADS : 0));
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        // last k-step: every wave has left stage kt's slots
        {
            const Src qa = src_a(kt + SA, a_slot);
            const Src qb2 = src_b(kt + 2, b_slot);  // SB = 2 only
            const char* nxt_a = lds + a_next * A_BYTES;
            const char* nxt_b = lds + b_next * B_BYTES;
            constexpr int C = (kKS - 1) & 1;
            constexpr int ND = A_LOADS + (SB == 2 ? B_LOADS : 0);
            static_for<0, NM>([&](auto ic) {
                constexpr int idx = decltype(ic)::value;
                constexpr int i = idx / FN, j = idx % FN;
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[C][i], fb[C][j], acc[i][j], 0, 0, 0);
                static_for<(ND * idx) / NM, (ND * (idx + 1)) / NM>([&](auto lc) {
                    constexpr int l = decltype(lc)::value;
                    if constexpr (l < A_LOADS)
                        lds_dma16_run<l>(qa.rsrc, a_off[l], qa.koff, qa.dst);
                    else
                        lds_dma16_run<l - A_LOADS>(qb2.rsrc, b_off[l - A_LOADS], qb2.koff, qb2.dst);
                });
                // first fragments of stage kt+1: early in the k-step, so they are back before its end
                static_for<2 * idx, (2 * idx + 2 < NR ? 2 * idx + 2 : NR)>([&](auto rc) {
                    constexpr int r = decltype(rc)::value;
                    if constexpr (r < FM)
                        fa[0][r] = *reinterpret_cast<const v4i*>(nxt_a + a_frag_off[r][0]);
                    else
                        fb[0][r - FM] = *reinterpret_cast<const v4i*>(nxt_b + b_frag_off[r - FM][0]);
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        }
        a_slot = a_next;
        b_slot = b_next;
    }

    // The last trips issued the (empty-descriptor) loads of stages KT and KT+1 into the rings; the abs-max
    // reduction below reuses the first bytes of the rings, so those loads must have landed (they return at
    // once: nothing is fetched) before anything else is written there.  Asm-issued loads are invisible to the
    // compiler's own wait insertion.
    if constexpr (kGen || (kEpi & 2) != 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));

    // Epilogue.  Accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4 and
    // column l%32 of its 32x32 block: 32 lanes store 128 contiguous bytes of one row.
    float next_scale = 0.0f;
    if (do_req) next_scale = ep.next_scale[0];
    unsigned amax = 0u;
    // A tile that lies wholly inside y (every tile of the BERT shapes) takes stores with a
    // per-lane column offset in a VGPR and the row offset in an SGPR: about six instructions
    // per element.  With one wave per SIMD the epilogue is bound by instruction issue, and
    // the bounds-checked path below costs twice as many.
    if (interior) {
        const int esize = do_req ? 1 : 4;
        const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(
            reinterpret_cast<char*>(ep.y) + tile_row0 * esize, 0, BM * N * esize, 0x00020000);
        const __amdgpu_buffer_rsrc_t racc = __builtin_amdgcn_make_buffer_rsrc(
            do_dump ? ep.acc_out + tile_row0 : ep.acc_out, 0, do_dump ? BM * N * 4 : 0, 0x00020000);
        // An fp32 y larger than a quarter of the 256 MB Infinity Cache is stored non-temporally:
        // it could not stay cached until its consumer runs anyway, and kept out it neither evicts
        // the next kernels' inputs nor leaves dirty lines to drain under them (whole BERT-Large
        // layer step 5-6 % faster; a GEMM timed alone with a cache-resident output does not show
        // it).  Smaller outputs are left for the cache to hand to their consumer.
        const bool stream_out = (int64_t)M * N * 4 > ((int64_t)64 << 20);
        float famax = 0.0f;
        if constexpr (kGen) fetch_first_residuals();
        auto store_tile = [&](auto ntc) {
        constexpr int kAux = decltype(ntc)::value ? 2 : 0;  // aux bit 1 = nt
        static_for<0, FN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int n = n0 + wn * TN + j * 32 + l32;
            const ColConst cc = ColConst{ep.bias ? quantize_bias(bias_col[j], sx, sw_col[j]) : 0, dequant_factor(sx, sw_col[j])};
            const int elem0 = row0 * N + n;
            static_for<0, FM>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                constexpr int b = j * FM + i;
                if constexpr (b + kResAhead < FM * FN) {
                    if (do_res) fetch_residual(std::integral_constant<int, b + kResAhead>{});
                }
                static_for<0, 16>([&](auto ec) {
                    constexpr int e = decltype(ec)::value;
                    constexpr int dm = i * 32 + 8 * (e >> 2) + (e & 3);
                    const int row_elems = dm * N;  // wave-uniform: lives in an SGPR
                    const int a = acc[i][j][e] + cc.bq;
                    float yv = (float)a * cc.r;
                    if (do_dump) __builtin_amdgcn_raw_buffer_store_b32((unsigned)a, racc, elem0 * 4, row_elems * 4, 0);
                    if (do_gelu) yv = gelu_erf(yv);
                    if (do_res) yv = __fadd_rn(yv, res[b % kResSlots][e]);
                    if (do_amax) famax = __builtin_fmaxf(famax, __builtin_fabsf(yv));  // one VALU op: |.| is a source modifier
                    if (do_req)
                        __builtin_amdgcn_raw_buffer_store_b8((unsigned char)quantize_code(yv, next_scale), ry, elem0,
                                                             row_elems, 0);
                    else
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(yv), ry, elem0 * 4, row_elems * 4, kAux);
                    // Keep the stores trickling out between the arithmetic of the next elements: left
                    // alone, the scheduler gathers 32 stores into one burst during which the VALU idles.
                    if constexpr ((e & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                });
            });
        });
        };
        if (stream_out && !do_req)
            store_tile(std::true_type{});
        else
            store_tile(std::false_type{});
        amax = __float_as_uint(famax);  // non-negative floats order like their bit patterns
    } else {
        static_for<0, FN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int n = n0 + wn * TN + j * 32 + l32;
            if (n < N) {
                const ColConst cc = ColConst{ep.bias ? quantize_bias(bias_col[j], sx, sw_col[j]) : 0, dequant_factor(sx, sw_col[j])};
                static_for<0, FM>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    const int mb = m0 + wm * TM + i * 32 + 4 * hi;
                    if constexpr (kPlain) {
                        float* yp = reinterpret_cast<float*>(ep.y) + (int64_t)mb * N + n;
                        static_for<0, 16>([&](auto ec) {
                            constexpr int e = decltype(ec)::value;
                            constexpr int dm = 8 * (e >> 2) + (e & 3);
                            if (mb + dm < M) yp[(int64_t)dm * N] = (float)(acc[i][j][e] + cc.bq) * cc.r;
                        });
                    } else {
                        static_for<0, 16>([&](auto ec) {
                            constexpr int e = decltype(ec)::value;
                            const int m = mb + 8 * (e >> 2) + (e & 3);
                            if (m < M) {
                                unsigned ab =
                                    epilogue_store(ep, (int64_t)m * N + n, acc[i][j][e] + cc.bq, cc.r, next_scale);
                                amax = max(amax, ab);
                            }
                        });
                    }
                });
            }
        });
    }
    if constexpr (kGen || (kEpi & 2) != 0) {
        if (do_amax) {  // one atomic max per workgroup; the stage buffers are dead by now
            unsigned* wave_amax = reinterpret_cast<unsigned*>(lds);
            __syncthreads();
            amax = wave_max_u32(amax);
            if (lane == 0) wave_amax[wave] = amax;
            __syncthreads();
            if (threadIdx.x == 0) {
#pragma unroll
                for (int w = 1; w < NW; ++w) amax = max(amax, wave_amax[w]);
                // The running maximum only grows, so a workgroup whose own maximum does not exceed
                // what is already there (read past the non-coherent L2) has nothing to add: after
                // the first few workgroups almost none issues the read-modify-write, which
                // serialises on one address.
                unsigned* slot = reinterpret_cast<unsigned*>(ep.out_amax);
                if (amax > __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(slot, amax);
            }
        }
    }
#endif
}

template <int BM, int BN, int WGM, int WGN, int SB>
int launch_tile(const int8_t* xq, const int8_t* wq, int M, int N, int K, int group_m, const Epilogue& ep,
                       hipStream_t st)
{
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const dim3 grid(tiles_m * tiles_n), block(WGM * WGN * 64);
#define Q8_LAUNCH_EPI(E)                                                                                         \
    hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WGM, WGN, SB, E>), grid, block, 0, st, xq, wq, M, N, K, tiles_n, \
                       group_m, ep)
    const int epi = (ep.acc_out != nullptr || ep.flags > 5u || (ep.residual && ep.flags)) ? -1 : ep.residual ? 8 : (int)ep.flags;
    switch (epi) {
        case 0: Q8_LAUNCH_EPI(0); break;
        case 1: Q8_LAUNCH_EPI(1); break;
        case 2: Q8_LAUNCH_EPI(2); break;
        case 3: Q8_LAUNCH_EPI(3); break;
        case 4: Q8_LAUNCH_EPI(4); break;
        case 5: Q8_LAUNCH_EPI(5); break;
        case 8: Q8_LAUNCH_EPI(8); break;
        default: Q8_LAUNCH_EPI(-1); break;
    }
#undef Q8_LAUNCH_EPI
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8
