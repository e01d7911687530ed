// Streaming and merge kernels of the matrix-core verify attention, and their launchers, as templates.
// Included by one translation unit per head grouping (attn_mfma_g1.hip ...), so that the many
// instances compile in parallel; attn_mfma.hip holds the plan kernel and the dispatch.
//
// Work decomposition.  The KV cache of one (request, KV head) pair ("unit") is a run of
// 16-token tiles, one per cache block.  All tiles of all units form one flat sequence (unit
// major).  A plan kernel writes that sequence out as a flat list of tile addresses (physical
// block * kv heads + kv head) and cuts it into `num_waves` contiguous spans of equal cost (a
// tile costs one, opening a unit costs a fixed number of tiles); every wavefront streams one
// span, so the load is balanced whatever the mix of context lengths, and the load side of the
// kernel is a plain linear walk that never stops at a unit boundary.  A span may cover the tail
// of one unit, several whole units and the head of another; for every unit it touches the wave
// has one partial result (softmax reference, sum, unnormalised output).  In the instances with
// at most two row blocks the four wavefronts of a workgroup, whose spans are consecutive, hand
// the partials of a shared unit from right to left through LDS and combine them by their
// log-sum-exp; a unit that lies inside one workgroup's spans is normalised, rounded and
// written by that workgroup.  What is left (a unit that crosses workgroups; every split unit
// in the other instances) goes to device memory as a partial in slot `workgroup + unit`
// (`wave + unit` without the LDS hand-over; unique along the sequence either way), and a last
// kernel merges those partials in span order and writes the rounded output.
//
// Per tile, with rows = (k+1) * (query heads per KV head) padded to a multiple of 16:
//   S^T[token][row] = K[token][:] . Q[row][:]   v_mfma_f32_16x16x32_bf16, K tile as A operand
//   online softmax on S^T in registers (a row's 16 scores sit in 4 lanes x 4 registers)
//   O^T[d][row]    += V[token][d] * P[row][token]   v_mfma_f32_16x16x16_bf16, P taken straight
//                     from the S^T accumulator layout, V as A operand
// Both K and V are read from HBM directly in operand layout with 16-byte loads: for K a lane
// holds 8 consecutive d of one token; for V a lane holds d = 8*i .. 8*i+7 of four tokens and
// the eight M-blocks of O^T are the eight interleaved d-phases, so no transpose through LDS is
// needed (only a 16-bit pack per operand register).
#pragma once

#include <type_traits>

#include <hip/hip_ext.h>

#include "common.h"
#include "span_cuts.h"
#include "tree_window.h"

namespace ss {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));

constexpr int D = kMfmaHeadDim;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSlack = 8.0f;       // log2 headroom of the lagging softmax reference
constexpr float kNoMax = -1.0e30f;   // reference before any score was seen (finite, so that -inf - ref stays -inf)
constexpr int kIdWindow = 512;       // tile addresses a wave stages in LDS at a time
constexpr int kMaxFlagPolls = 1 << 23;   // polls of a neighbour's deposit flag before giving up (each at least 128 cycles)
constexpr int kPartRowStride = 33;   // float4 per staged partial row in LDS (32 of data + 1 of padding)
template <int NB>
constexpr bool kChainMerge = NB <= 2;   // instances that combine the spans of a workgroup in LDS
template <int NB>
constexpr bool kStageRows = NB <= 4;    // instances that write partials as whole rows through LDS (measured: with five
                                        // row blocks the staging costs more than the scattered stores it replaces)

// ---------------------------------------------------------------------------------------------
// streaming kernel
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t pack_hi16(uint32_t lo_src, uint32_t hi_src)
{
    // (hi_src & 0xffff0000) | (lo_src >> 16): upper halves of two words
    return __builtin_amdgcn_perm(hi_src, lo_src, 0x07060302u);
}
__device__ __forceinline__ uint32_t pack_lo16(uint32_t lo_src, uint32_t hi_src)
{
    return __builtin_amdgcn_perm(hi_src, lo_src, 0x05040100u);
}

// 8 e4m3 bytes (two words) -> 8 bf16 (exact: e4m3 has 4 significant bits)
__device__ __forceinline__ uint4 fp8x8_to_bf16x8(uint32_t w0, uint32_t w1)
{
    const float2v a = __builtin_amdgcn_cvt_pk_f32_fp8(w0, false);
    const float2v b = __builtin_amdgcn_cvt_pk_f32_fp8(w0, true);
    const float2v c = __builtin_amdgcn_cvt_pk_f32_fp8(w1, false);
    const float2v d = __builtin_amdgcn_cvt_pk_f32_fp8(w1, true);
    uint4 r;
    r.x = pack_hi16(__float_as_uint(a.x), __float_as_uint(a.y));
    r.y = pack_hi16(__float_as_uint(b.x), __float_as_uint(b.y));
    r.z = pack_hi16(__float_as_uint(c.x), __float_as_uint(c.y));
    r.w = pack_hi16(__float_as_uint(d.x), __float_as_uint(d.y));
    return r;
}

// KV tiles are read exactly once per call: non-temporal loads keep them from displacing what is reused
// (partials, queries, the tile list) in the caches.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 stream_load16(const char *p)
{
    const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ uint2 stream_load8(const char *p)
{
    const u32x2 r = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
    return make_uint2(r.x, r.y);
}

// Output accumulators live in the accumulator registers (the matrix instructions are selected in that form
// once a kernel needs more than 256 registers).  A value that ordinary vector arithmetic produced -- the zero
// of a new unit, a rescaled or merged accumulator -- is handed over through this empty statement, so that
// every value flowing into the tile loop comes from an accumulator register; otherwise the compiler keeps the
// loop-carried accumulators in vector registers and moves all of them to the accumulator file and back on
// every tile.
__device__ __forceinline__ void to_accumulator_file(float4v &c) { asm volatile("" : "+a"(c)); }
// The opposite direction for the rare rescale: the move is written out, so that it stays inside the rarely taken
// branch (left to the compiler, the moves of all accumulators to vector registers can end up in front of the
// branch, on every tile).  The compiler does not look into the statement: the caller leaves the wait states
// between the last matrix instruction that wrote the register and this read (accumulator_read_guard).
__device__ __forceinline__ float from_accumulator_file(float x)
{
    float r;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(x));
    return r;
}
__device__ __forceinline__ void accumulator_read_guard() { asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory"); }

template <bool FP8>
struct TileRegs {
    // bf16: k[ks] = 8 bf16 of token (lane&15) at d = 32*ks + 8*(lane>>4)
    // fp8 : k[kk] = 16 bytes of token (lane&15) at d = 64*kk + 16*(lane>>4)   (kk = 0,1)
    uint4 k[FP8 ? 2 : 4];
    // bf16: v[e] = 8 bf16 of token 4*(lane>>4)+e at d = 8*(lane&15)
    // fp8 : v[e] = 8 bytes of the same
    typename std::conditional<FP8, uint2, uint4>::type v[4];
    float ks, vs;  // block scales (fp8), 1 otherwise
};

// All loads of one tile are vector loads issued back to back, so one counter orders them and the
// consumer can wait for exactly this tile.  `addr` = physical block * kv heads + kv head indexes
// both the 4 KB (2 KB for e4m3) tile and its scale.  `vzero` is a lane register holding 0 that the
// compiler cannot see through: it keeps the (wave-uniform) scale reads on the vector path too.
template <bool FP8>
__device__ __forceinline__ void load_tile(TileRegs<FP8> &t, const AttnArgs &a, const float *__restrict__ k_scale,
                                          const float *__restrict__ v_scale, int addr, int lane, int vzero)
{
    constexpr int ES = FP8 ? 1 : 2;
    const int64_t blk = (int64_t)addr * (kTile * D * ES);
    const char *kp = static_cast<const char *>(a.k) + blk + (lane & 15) * (D * ES) + (lane >> 4) * 16;
    const char *vp = static_cast<const char *>(a.v) + blk + (lane >> 4) * (4 * D * ES) + (lane & 15) * (8 * ES);
#pragma unroll
    for (int i = 0; i < (FP8 ? 2 : 4); ++i) t.k[i] = stream_load16(kp + i * 64);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if constexpr (FP8)
            t.v[e] = stream_load8(vp + e * (D * ES));
        else
            t.v[e] = stream_load16(vp + e * (D * ES));
    }
    if constexpr (FP8) {
        t.ks = k_scale[addr + vzero];
        t.vs = v_scale[addr + vzero];
    } else {
        t.ks = 1.f;
        t.vs = 1.f;
    }
}

// NB    16-row blocks of query rows the kernel is compiled for (covers max_q_len * G rows)
// NBUF  KV tiles resident per wave: one being consumed, NBUF-1 in flight from HBM
// QLDS  keep the query operands in LDS (in operand order, one 1 KB line per row block and k-step)
//       instead of registers: for many row blocks the registers are needed for the accumulators
// TREE  the new tokens of a request form a draft tree: a row's visibility among them comes from its
//       mask word instead of the chain's "tokens up to my own"
template <int G, int NB, bool FP8, int NBUF, bool QLDS, bool TREE>
__global__ __launch_bounds__(64 * kWavesPerWg, 1) void attn_stream_kernel(
    AttnArgs a, const int32_t *__restrict__ tile_addr, const int32_t *__restrict__ wave_desc,
    const int32_t *__restrict__ tile_prefix,
    const int32_t *__restrict__ kv_len, const int32_t *__restrict__ q_indptr, const float *__restrict__ k_scale,
    const float *__restrict__ v_scale)
{
    // The metadata arrays come in as separate no-alias arguments so that their wave-uniform reads
    // become scalar loads (own counter, no ordering against the vector KV loads).
    __shared__ int32_t id_lds[kWavesPerWg][kIdWindow];
    __shared__ uint4 q_lds[QLDS ? kWavesPerWg * NB * 4 * 64 : 1];
    // one 16-row block of a partial per wave, rows 33 float4 apart (the odd stride spreads the rows over the banks)
    __shared__ float4v o_lds[kStageRows<NB> ? kWavesPerWg : 1][kStageRows<NB> ? 16 * kPartRowStride : 1];
    __shared__ float2 ml_lds[kWavesPerWg][16];
    // CHAIN: the wavefronts of a workgroup own consecutive spans, so a unit that runs on from one span into the
    // next is combined inside the workgroup: the right-hand wave leaves the result of its part in its deposit
    // slot, the left-hand one folds it into its own.  Only what crosses a workgroup's edge goes to memory as a
    // partial; a unit that lies inside one workgroup is finished here.
    // (Only for one or two row blocks: with three the deposit slots take 100 KB and the ragged workload, the one
    // that uses them, ran 7 % slower; beyond that the queries live in LDS and there is no room.)
    constexpr bool CHAIN = kChainMerge<NB>;
    __shared__ float4v dep_o[CHAIN ? kWavesPerWg : 1][CHAIN ? NB * 16 * kPartRowStride : 1];
    __shared__ float2 dep_ml[CHAIN ? kWavesPerWg : 1][CHAIN ? NB * 16 : 1];
    __shared__ int dep_flag[kWavesPerWg];   // 0 nothing yet; 1 deposited; 2 deposited and it reaches the unit's last tile
    const int lane = threadIdx.x & 63;
    const int wslot = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wave = blockIdx.x * kWavesPerWg + wslot;
    const int r16 = lane & 15, jq = lane >> 4;
    int vzero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
    int32_t *ids = id_lds[wslot];
    uint4 *qs = q_lds + (QLDS ? wslot * NB * 4 * 64 : 0) + (QLDS ? lane : 0);

    // where this wave's span starts: written by the plan kernel (waves past the partition count get x0 == x1)
    int b, g, tile, nb_tiles;
    long long x0, x1;
    int meta_L, meta_q0, meta_q1, meta_nbt;   // kv_len / q_indptr / tile count of the next unit to open
    int desc_addr[kDescAddrs];
    {
        const int32_t *d = wave_desc + (long long)wave * kDescInts;
        b = d[0]; g = d[1]; tile = d[2]; nb_tiles = d[3];
        x0 = d[4]; x1 = d[5];
        meta_L = d[6]; meta_q0 = d[7]; meta_q1 = d[8]; meta_nbt = nb_tiles;
#pragma unroll
        for (int j = 0; j < kDescAddrs; ++j) desc_addr[j] = d[9 + j];
    }
    static_assert(NBUF - 1 <= kDescAddrs, "descriptor carries too few tile addresses");
    if (lane == 0) dep_flag[wslot] = 0;
    __syncthreads();   // the only barrier: every wave's flag is clear before any neighbour can look at it
    if (x0 >= x1) return;

    // ---- state of the unit being computed ----
    int span_left = (int)(x1 - x0);   // tiles of the span not yet computed
    int seg_left = 0;                 // of those, tiles that still belong to the current unit
    int seg_tile0 = 0;                // the unit's tile the current segment began with
    int L = 0, q0 = 0, q_len = 0, rows = 0, nbu = 0;   // nbu: 16-row blocks the unit really has (for its partial)
    bf16x8 qreg[QLDS ? 1 : NB][4];    // Q as B operand: lane holds row 16*nb + r16, 8 consecutive d per k-step
    int lim[TREE ? 1 : NB];           // chain: last visible cache position of this lane's row in block nb
    uint32_t newmask[TREE ? NB : 1];  // tree: which new tokens of the request the lane's row attends
    int ctx = 0;                      // cache positions before the unit's new tokens
    float m_run[NB], l_run[NB];
    float4v acc[8][NB];
    const float sc2 = a.sm_scale * kLog2e;

    // (the metadata of the unit after the current one is fetched a unit ahead)
    auto begin_unit_issue = [&]() __attribute__((always_inline)) {
        L = meta_L;
        q0 = meta_q0;
        q_len = meta_q1 - meta_q0;
        const int q_here = window_q_len(q_len, a.q_lo, a.q_win);   // query tokens of this pass's window
        nb_tiles = meta_nbt;
        rows = q_here * G;
        nbu = (rows + 15) >> 4;
        ctx = L - q_len;
        {
            const int nb_ = (g + 1 == a.num_kv_heads) ? b + 1 : b;   // request of the next unit
            if (nb_ != b && nb_ < a.batch) {
                meta_L = kv_len[nb_];
                meta_q0 = q_indptr[nb_];
                meta_q1 = q_indptr[nb_ + 1];
                meta_nbt = tile_prefix[nb_ + 1] - tile_prefix[nb_];
            }
        }
        seg_left = nb_tiles - tile < span_left ? nb_tiles - tile : span_left;
        seg_tile0 = tile;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int n = nb * 16 + r16;
            const bool ok = n < rows;
            const int qi = a.q_lo + n / G, hh = n % G;   // query token within the request, head within the group
            if constexpr (TREE)   // padding rows see every new token: harmless, and no row is empty
                newmask[nb] = ok ? a.tree_mask[q0 + qi] : (2u << (q_len - 1)) - 1u;
            else
                lim[nb] = ok ? L - q_len + qi : L - 1;
            const char *qp = static_cast<const char *>(a.q) +
                             (((long long)(q0 + qi) * a.num_q_heads + g * G + hh) * D) * 2;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int d0 = FP8 ? ((ks >> 1) * 64 + jq * 16 + (ks & 1) * 8) : (ks * 32 + jq * 8);
                uint4 w = make_uint4(0, 0, 0, 0);
                if (ok) w = *reinterpret_cast<const uint4 *>(qp + d0 * 2);
                if constexpr (QLDS)
                    qs[(nb * 4 + ks) * 64] = w;
                else
                    qreg[nb][ks] = __builtin_bit_cast(bf16x8, w);
            }
            m_run[nb] = kNoMax;
            l_run[nb] = 0.f;
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) {
                acc[mb][nb] = float4v{0.f, 0.f, 0.f, 0.f};
                to_accumulator_file(acc[mb][nb]);
            }
        }
    };
    // Have the queries arrive here, inside the rarely taken branch, so that the steady-state path
    // never carries a pending load of them.
    auto begin_unit_wait = [&]() __attribute__((always_inline)) {
        if constexpr (!QLDS) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(qreg[nb][ks]));
        }
        if constexpr (TREE) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+v"(newmask[nb]));
        }
    };

    // A segment (the part of a unit that lies in this span) has ended: `starts` / `ends` say whether it holds
    // the unit's first / last tile.
    auto end_unit = [&](bool starts, bool ends) __attribute__((always_inline)) {
        // The accumulators were last written by MFMAs in another basic block: give them the wait
        // states a read needs before anything below touches them.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
        float lsum[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float l = l_run[nb];
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            lsum[nb] = l;
        }
        bool to_end = ends;   // does the result held here reach the unit's last tile?
        if constexpr (CHAIN) {
            if (!ends && wslot + 1 < kWavesPerWg) {
                // The unit runs on into the right-hand neighbour's span, where it is that wave's first
                // segment: finished long ago unless the spans are very short.  Fold its result into mine
                // (mine first: a fixed order, so the bits do not depend on timing).
                // (relaxed LDS accesses: a volatile or acquiring load would first wait for every tile in flight)
                // The wait is bounded (about a second): the neighbour is a wave of the same workgroup and reaches its
                // deposit without waiting for anything itself, so the bound is never met; if it ever were, the unit's
                // rows come out as NaN instead of the kernel hanging.
                int f = __hip_atomic_load(&dep_flag[wslot + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                for (int polls = 0; f == 0 && polls < kMaxFlagPolls; ++polls) {
                    __builtin_amdgcn_s_sleep(2);
                    f = __hip_atomic_load(&dep_flag[wslot + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                if (f == 0) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) lsum[nb] = __builtin_nanf("");
                }
                to_end = f == 2;
                // (the deposit is read after the flag: the hardware serves a wave's LDS requests in order; this
                // keeps the compiler from moving the reads ahead of the loop, at no instruction)
                asm volatile("" ::: "memory");
                const float4v *dq = dep_o[wslot + 1];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    if (nb < nbu) {
                        const float2 ml2 = dep_ml[wslot + 1][nb * 16 + r16];
                        const float m_new = fmaxf(m_run[nb], ml2.x);
                        const float wa = exp2f(m_run[nb] - m_new), wb = exp2f(ml2.x - m_new);
                        lsum[nb] = lsum[nb] * wa + ml2.y * wb;
                        m_run[nb] = m_new;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float4v lo = dq[(nb * 16 + r16) * kPartRowStride + jq * 8 + e * 2];
                            const float4v hi = dq[(nb * 16 + r16) * kPartRowStride + jq * 8 + e * 2 + 1];
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                acc[c][nb][e] = acc[c][nb][e] * wa + lo[c] * wb;
                                acc[4 + c][nb][e] = acc[4 + c][nb][e] * wa + hi[c] * wb;
                            }
                        }
                    }
                }
            }
            if (!starts && wslot > 0) {
                // The unit began in the left-hand neighbour's span: leave the result for it.
                float4v *dq = dep_o[wslot];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    if (nb < nbu) {
                        if (jq == 0) dep_ml[wslot][nb * 16 + r16] = make_float2(m_run[nb], lsum[nb]);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float4v lo = {acc[0][nb][e], acc[1][nb][e], acc[2][nb][e], acc[3][nb][e]};
                            const float4v hi = {acc[4][nb][e], acc[5][nb][e], acc[6][nb][e], acc[7][nb][e]};
                            dq[(nb * 16 + r16) * kPartRowStride + jq * 8 + e * 2] = lo;
                            dq[(nb * 16 + r16) * kPartRowStride + jq * 8 + e * 2 + 1] = hi;
                        }
                    }
                }
                // The slot's contents are in LDS before the flag says so: LDS serves a wave's requests in order,
                // and the wait below covers LDS only (a release fence would also wait for the tiles in flight).
                asm volatile("" ::: "memory");        // (the compiler keeps the deposit's stores above this line)
                __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
                __builtin_amdgcn_wave_barrier();
                asm volatile("" ::: "memory");
                if (lane == 0) __hip_atomic_store(&dep_flag[wslot], to_end ? 2 : 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                return;
            }
        }
        // What is held here goes to memory: as the finished output if it covers the whole unit, else as a
        // partial in slot (workgroup, or wave without CHAIN) + unit, unique along the tile sequence.
        const bool whole = CHAIN && starts && to_end;
        const long long slot = (long long)(CHAIN ? (int)blockIdx.x : wave) + (long long)b * a.num_kv_heads + g;
        float *po = a.part_o + slot * a.rows_pad * D;
        float *pml = a.part_ml + slot * a.rows_pad * 2;
        // A lane holds 32 consecutive d of one row (d = 32*jq + 8*e + mb), in registers that are 16 bytes
        // apart in memory: written directly, every store would scatter 16-byte pieces over 64 cache lines.
        // The block goes through LDS instead and leaves as whole rows, two per store (kStageRows).
        float4v *ol = o_lds[kStageRows<NB> ? wslot : 0];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (nb < nbu) {
                const int n = nb * 16 + r16;
                if (whole) {
                    if (jq == 0) ml_lds[wslot][r16] = make_float2(m_run[nb], lsum[nb]);
                } else if (n < rows && jq == 0) {
                    pml[n * 2 + 0] = m_run[nb];
                    pml[n * 2 + 1] = lsum[nb];
                }
                if constexpr (!kStageRows<NB>) {
                    if (n < rows) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {   // accumulator row 4*jq+e of M-block mb is d = 8*(4*jq+e) + mb
                            float *dst = po + n * D + (jq * 4 + e) * 8;
                            const float4v lo = {acc[0][nb][e], acc[1][nb][e], acc[2][nb][e], acc[3][nb][e]};
                            const float4v hi = {acc[4][nb][e], acc[5][nb][e], acc[6][nb][e], acc[7][nb][e]};
                            *reinterpret_cast<float4v *>(dst) = lo;
                            *reinterpret_cast<float4v *>(dst + 4) = hi;
                        }
                    }
                    continue;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // accumulator row 4*jq+e of M-block mb is d = 8*(4*jq+e) + mb
                    const float4v lo = {acc[0][nb][e], acc[1][nb][e], acc[2][nb][e], acc[3][nb][e]};
                    const float4v hi = {acc[4][nb][e], acc[5][nb][e], acc[6][nb][e], acc[7][nb][e]};
                    ol[r16 * kPartRowStride + jq * 8 + e * 2] = lo;
                    ol[r16 * kPartRowStride + jq * 8 + e * 2 + 1] = hi;
                }
                __builtin_amdgcn_wave_barrier();
                // same wave, LDS keeps program order: no barrier.  All rows are read back first, in straight-line
                // code, so that the LDS latency is paid once and not in front of every store.
                float4v rowv[8];
                float2 rowml[8];
#pragma unroll
                for (int it = 0; it < 8; ++it) {
                    const int row = it * 2 + (lane >> 5);
                    rowv[it] = ol[row * kPartRowStride + (lane & 31)];
                    if (whole) rowml[it] = ml_lds[wslot][row];
                }
#pragma unroll
                for (int it = 0; it < 8; ++it) {
                    const int row = it * 2 + (lane >> 5), nn = nb * 16 + row;
                    const float4v v = rowv[it];
                    if (whole) {
                        // normalise, round to bf16 (nearest even), 256-byte output rows; lse from the row's (m, l)
                        const float2 ml = rowml[it];
                        const float inv = 1.f / ml.y;
                        const int qi = a.q_lo + nn / G, hh = nn % G;
                        const long long orow = (long long)(q0 + qi) * a.num_q_heads + g * G + hh;
                        const float2v lo2 = {v[0] * inv, v[1] * inv}, hi2 = {v[2] * inv, v[3] * inv};
                        uint2 pk;
                        pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo2, bf16x2));
                        pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi2, bf16x2));
                        if (nn < rows) {
                            *reinterpret_cast<uint2 *>(static_cast<__bf16 *>(a.out) + orow * D + (lane & 31) * 4) = pk;
                            if (a.lse && (lane & 31) == 0) a.lse[orow] = (ml.x + log2f(ml.y)) * kLn2;
                        }
                    } else if (nn < rows) {
                        *reinterpret_cast<float4v *>(po + nn * D + (lane & 31) * 4) = v;
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    };
    // (b, g) <- the unit after it (its metadata is already in meta_*)
    auto next_unit = [&]() __attribute__((always_inline)) {
        tile = 0;
        if (++g == a.num_kv_heads) {
            g = 0;
            ++b;
        }
    };

    // One tile: S^T = K Q^T for all row blocks, softmax, O^T += V^T P^T.  Row blocks beyond the
    // unit's rows hold zero queries; they are computed anyway (cheaper than branching, which was
    // measured) and never stored.  Three wave-uniform branches leave the straight line: the mask
    // selects (only tiles that reach into the request's new tokens), the clearing of V slots past the
    // end of the cache (e4m3 instances: only a cache's last tile) and the rare rescale.  The compiler
    // keeps the wait states between a matrix instruction and the first read of its result, also across
    // these branches; where the read is written out by hand (the rescale, from_accumulator_file) or
    // follows a scheduling barrier (the end of a unit), explicit wait states stand in front of it.
    // The order of the pieces is chosen so that vector work that does not depend on a matrix result
    // follows each group of MFMAs: the V operands are built while S^T is in the matrix pipeline, and
    // a row block's exponentials while the previous block's output MFMAs run.
    auto compute = [&](const TileRegs<FP8> &t, int ti) __attribute__((always_inline)) {
        const int tok0 = ti * kTile + jq * 4;   // first of this lane's four cache positions

        bf16x8 kop[4];
        if constexpr (FP8) {
            kop[0] = __builtin_bit_cast(bf16x8, fp8x8_to_bf16x8(t.k[0].x, t.k[0].y));
            kop[1] = __builtin_bit_cast(bf16x8, fp8x8_to_bf16x8(t.k[0].z, t.k[0].w));
            kop[2] = __builtin_bit_cast(bf16x8, fp8x8_to_bf16x8(t.k[1].x, t.k[1].y));
            kop[3] = __builtin_bit_cast(bf16x8, fp8x8_to_bf16x8(t.k[1].z, t.k[1].w));
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) kop[ks] = __builtin_bit_cast(bf16x8, t.k[ks]);
        }
        float4v s[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) s[nb] = float4v{0.f, 0.f, 0.f, 0.f};
        if constexpr (QLDS) {
            // operands come from LDS a few MFMAs ahead of their use, so that its latency is covered
            constexpr int NOPS = 4 * NB, AHEAD = NOPS < 6 ? NOPS : 6;
            uint4 qb[AHEAD];
#pragma unroll
            for (int i = 0; i < AHEAD; ++i) qb[i] = qs[((i % NB) * 4 + i / NB) * 64];
#pragma unroll
            for (int i = 0; i < NOPS; ++i) {
                const int ks = i / NB, nb = i % NB;
                const bf16x8 qop = __builtin_bit_cast(bf16x8, qb[i % AHEAD]);
                if (i + AHEAD < NOPS) {
                    const int i2 = i + AHEAD;
                    qb[i % AHEAD] = qs[((i2 % NB) * 4 + i2 / NB) * 64];
                }
                s[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[ks], qop, s[nb], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    s[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[ks], qreg[nb][ks], s[nb], 0, 0, 0);
        }

        // V operand registers: vop[mb] = d-phase mb of tokens tok0 .. tok0+3.
        short4v vop[8];
#pragma unroll
        for (int h = 0; h < 4; ++h) {   // word h of each token's 8 values holds d-phases 2h and 2h+1
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (FP8) {
                    const uint32_t src = (h < 2) ? t.v[e].x : t.v[e].y;   // two e4m3 bytes -> two bf16, exact
                    const float2v f = (h & 1) ? __builtin_amdgcn_cvt_pk_f32_fp8(src, true)
                                              : __builtin_amdgcn_cvt_pk_f32_fp8(src, false);
                    w[e] = pack_hi16(__float_as_uint(f.x), __float_as_uint(f.y));
                } else {
                    w[e] = (&t.v[e].x)[h];
                }
            }
            uint2 lo, hi;
            lo.x = pack_lo16(w[0], w[1]);
            lo.y = pack_lo16(w[2], w[3]);
            hi.x = pack_hi16(w[0], w[1]);
            hi.y = pack_hi16(w[2], w[3]);
            vop[2 * h] = __builtin_bit_cast(short4v, lo);
            vop[2 * h + 1] = __builtin_bit_cast(short4v, hi);
        }
        // Slots at or past kv_len may hold anything (NaN, inf): they are cleared so that 0 * garbage cannot
        // occur.  Only the last tile of a cache has such slots; the e4m3 instances, which are bound by their
        // vector instructions, test for it (wave-uniform), the others clear unconditionally (measured: there the
        // branch costs more than the sixteen ANDs).
        if (!FP8 || ti * kTile + kTile > L) {
            const uint32_t m01 = (tok0 + 0 < L ? 0x0000ffffu : 0u) | (tok0 + 1 < L ? 0xffff0000u : 0u);
            const uint32_t m23 = (tok0 + 2 < L ? 0x0000ffffu : 0u) | (tok0 + 3 < L ? 0xffff0000u : 0u);
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) {
                uint2 w = __builtin_bit_cast(uint2, vop[mb]);
                w.x &= m01;
                w.y &= m23;
                vop[mb] = __builtin_bit_cast(short4v, w);
            }
        }

        // Online softmax with a lagging reference: p = 2^(s - m_ref).  The reference only moves
        // (and the accumulators are rescaled) when some score exceeds it by more than kSlack, so
        // p <= 2^kSlack and the common tile needs no cross-lane traffic and no rescale.  The common path forms
        // the exponent's argument with one fused multiply-add per score and tests all of them against the slack
        // at once; the scores themselves are only formed on the rare path (before a unit's first tile the
        // reference is so low that the argument has absorbed them).
        const float kscale = sc2 * t.ks;
        float pd[NB][4];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) pd[nb][e] = __builtin_fmaf(s[nb][e], kscale, -m_run[nb]);
        // Every row sees all of the context before the request's new tokens, so only the last tile or two of a
        // unit need the selects: the wave-uniform test skips them for the rest.
        const bool tail = ti * kTile + kTile > ctx;
        if (tail) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if constexpr (TREE) {
                    // Positions past the cache end are past the mask's last set bit.
                    const uint32_t vis = tree_visible4(newmask[nb], tok0 - ctx);
#pragma unroll
                    for (int e = 0; e < 4; ++e) pd[nb][e] = ((vis >> e) & 1u) ? pd[nb][e] : -INFINITY;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)   // causal limit among the new tokens / end of the cache
                        pd[nb][e] = (tok0 + e > lim[nb]) ? -INFINITY : pd[nb][e];
                }
            }
        }
        float top = pd[0][0];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) top = fmaxf(top, pd[nb][e]);
        if (__any(top > kSlack)) {
            accumulator_read_guard();
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                float sv[4];   // the scores, masked where the argument was
#pragma unroll
                for (int e = 0; e < 4; ++e) sv[e] = pd[nb][e] == -INFINITY ? -INFINITY : s[nb][e] * kscale;
                float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[nb], mx);
                const float alpha = __builtin_amdgcn_exp2f(m_run[nb] - m_new);
                l_run[nb] *= alpha;
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) {
                    const float4v c = acc[mb][nb];
                    float4v r = {from_accumulator_file(c[0]) * alpha, from_accumulator_file(c[1]) * alpha,
                                 from_accumulator_file(c[2]) * alpha, from_accumulator_file(c[3]) * alpha};
                    to_accumulator_file(r);
                    acc[mb][nb] = r;
                }
                m_run[nb] = m_new;
#pragma unroll
                for (int e = 0; e < 4; ++e) pd[nb][e] = sv[e] - m_new;
            }
        }
        if constexpr (NB >= 3) {
            // A wavefront issues in order: matrix instructions that stand back to back leave the vector ALU idle
            // while they run, and the vector work of a row block leaves the matrix pipeline idle.  With many row
            // blocks the kernel is bound by that, not by memory, so the blocks are software-pipelined by hand: the
            // exponentials and the packing of block nb+1 are cut into pieces of two or three instructions, one after
            // each of block nb's eight output MFMAs, and a scheduling barrier after every piece keeps the compiler
            // from gathering the matrix instructions together again.
            float pe[4];
            uint2 pk;
            auto piece = [&](int nb, int i) __attribute__((always_inline)) {
                if (i == 0) pe[0] = __builtin_amdgcn_exp2f(pd[nb][0]);
                if (i == 1) pe[1] = __builtin_amdgcn_exp2f(pd[nb][1]);
                if (i == 2) pe[2] = __builtin_amdgcn_exp2f(pd[nb][2]);
                if (i == 3) pe[3] = __builtin_amdgcn_exp2f(pd[nb][3]);
                if (i == 4) l_run[nb] += (pe[0] + pe[1]) + (pe[2] + pe[3]);
                if (i == 5) {
                    const float2v lo = {pe[0] * t.vs, pe[1] * t.vs};
                    pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
                }
                if (i == 6) {
                    const float2v hi = {pe[2] * t.vs, pe[3] * t.vs};
                    pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
                }
            };
#pragma unroll
            for (int i = 0; i < 7; ++i) piece(0, i);
            short4v pop = __builtin_bit_cast(short4v, pk);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) {
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vop[mb], pop, acc[mb][nb], 0, 0, 0);
                    if (nb + 1 < NB) {
                        piece(nb + 1, mb);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (nb + 1 < NB) pop = __builtin_bit_cast(short4v, pk);
            }
        } else {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                float p[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(pd[nb][e]);
                l_run[nb] += (p[0] + p[1]) + (p[2] + p[3]);
                const float2v lo = {p[0] * t.vs, p[1] * t.vs}, hi = {p[2] * t.vs, p[3] * t.vs};
                uint2 pk;
                pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
                pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
                const short4v pop = __builtin_bit_cast(short4v, pk);
#pragma unroll
                for (int mb = 0; mb < 8; ++mb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vop[mb], pop, acc[mb][nb], 0, 0, 0);
            }
        }
    };

    // one step of the compute side: consume a tile; at the end of a unit segment write its partial
    // and open the next segment (its query loads go out ahead of the next KV prefetch)
    auto step = [&](const TileRegs<FP8> &t) __attribute__((always_inline)) {
        compute(t, tile);
        ++tile;
        --span_left;
        if (--seg_left == 0) {
            end_unit(seg_tile0 == 0, tile == nb_tiles);
            next_unit();
            if (span_left > 0) {
                begin_unit_issue();
                begin_unit_wait();
            }
        }
    };

    // ---- load side: a linear walk over the span's tile addresses, staged in LDS a window at a time ----
    bool first_window = true;
    for (long long c0 = x0; c0 < x1; c0 += kIdWindow) {
        const int n = (int)(x1 - c0 < kIdWindow ? x1 - c0 : kIdWindow);
        // the window's addresses: vector reads now, into LDS once they have arrived
        int idtmp[kIdWindow / 64];
#pragma unroll
        for (int i = 0; i < kIdWindow / 64; ++i) idtmp[i] = (i * 64 + lane < n) ? tile_addr[c0 + i * 64 + lane] : 0;
        // the first NBUF-1 tiles do not wait for that: their addresses come by scalar reads
        int first_addr[NBUF - 1];
#pragma unroll
        for (int j = 0; j < NBUF - 1; ++j)
            first_addr[j] = first_window ? desc_addr[j] : tile_addr[c0 + (j < n ? j : n - 1)];
        if (first_window) begin_unit_issue();   // queries of the first unit go out before any KV tile

        TileRegs<FP8> buf[NBUF];
#pragma unroll
        for (int j = 0; j < NBUF - 1; ++j)
            if (j < n) load_tile<FP8>(buf[j], a, k_scale, v_scale, first_addr[j], lane, vzero);
        if (first_window) begin_unit_wait();
        first_window = false;
#pragma unroll
        for (int i = 0; i < kIdWindow / 64; ++i) ids[i * 64 + lane] = idtmp[i];

        int p_load = NBUF - 1;   // next tile of the window to load
        int id_v = ids[p_load < n ? p_load : n - 1];   // its address, read from LDS one step ahead of its use
        auto issue = [&](TileRegs<FP8> &t) __attribute__((always_inline)) {
            const int addr = __builtin_amdgcn_readfirstlane(id_v);
            ++p_load;
            id_v = ids[p_load < n ? p_load : n - 1];
            load_tile<FP8>(t, a, k_scale, v_scale, addr, lane, vzero);
        };

        // Software pipeline over a ring of NBUF tile buffers (fully unrolled: static registers).
        // The steady-state loop issues its prefetch unconditionally, so the wait before each
        // compute only covers the tile it needs and NBUF-1 tiles stay in flight; the last few
        // tiles of a window (and short windows) run through a conditional epilogue.
        int p = 0;
        for (; p + 2 * NBUF - 2 < n; p += NBUF) {
#pragma unroll
            for (int j = 0; j < NBUF; ++j) {
                issue(buf[(j + NBUF - 1) % NBUF]);
                __builtin_amdgcn_sched_barrier(0);  // keep the prefetch ahead of every use of the current tile
                step(buf[j]);
            }
        }
        // here buf[j] holds tile p + j for j < NBUF-1 (as far as such tiles exist)
#pragma unroll
        for (int j = 0; j < 2 * NBUF - 2; ++j) {
            if (p + j < n) {
                if (p + j + NBUF - 1 < n) issue(buf[(j + NBUF - 1) % NBUF]);
                step(buf[j % NBUF]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// merge: workgroup (unit, slab) combines the partials of 8 query rows of one unit
// ---------------------------------------------------------------------------------------------
constexpr int kMergeRows = 8;

template <int G>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a)
{
    const int slabs = a.rows_pad / kMergeRows;
    const int unit = blockIdx.x / slabs, slab = blockIdx.x % slabs;
    const int b = unit / a.num_kv_heads, g = unit % a.num_kv_heads;
    const int q0 = a.q_indptr[b];
    const int rows = window_q_len(a.q_indptr[b + 1] - q0, a.q_lo, a.q_win) * G;   // rows of this pass's window
    const int n = slab * kMergeRows + (threadIdx.x >> 5), d4 = threadIdx.x & 31;
    if (n >= rows) return;
    const long long total = a.plan->total_tiles;
    const long long nw = a.plan->num_waves;
    const int pre = a.tile_prefix[b];
    const int nb_tiles = a.tile_prefix[b + 1] - pre;
    const long long off = (long long)pre * a.num_kv_heads + (long long)g * nb_tiles;
    // The spans were cut at w*total_w/nw in the weighted coordinate (every unit: `weight` virtual tiles, then
    // its own); the last wave whose cut lies at or before coordinate t is ((t+1)*nw - 1) / total_w.  A cut
    // inside the unit's virtual part starts at its first tile, so the unit's first wave is the last one at
    // or before the end of that part, its last wave the last one before the next unit's stretch.
    SpanCuts cuts;
    cuts.prefix = a.tile_prefix;
    cuts.batch = a.batch;
    cuts.hkv = a.num_kv_heads;
    cuts.weight = a.plan->unit_weight;
    cuts.total = total;
    cuts.total_w = total + (long long)cuts.weight * a.batch * a.num_kv_heads;
    cuts.nw = nw;
    int w_first, w_last;
    cuts.unit_waves(off + (long long)cuts.weight * unit, nb_tiles, w_first, w_last);
    if (a.chain) {
        // the streaming kernel has combined the spans of each workgroup: one partial per workgroup the unit
        // touches, and a unit inside a single workgroup is already finished
        w_first /= kWavesPerWg;
        w_last /= kWavesPerWg;
        if (w_first == w_last) return;
    }

    // running merge: (m, l, o) <- (m, l, o) (+) partial, both relative to their own reference m
    float m_all = kNoMax, l_all = 0.f;
    float4v o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int w = w_first; w <= w_last; ++w) {
        const long long row = ((long long)w + unit) * a.rows_pad + n;
        const float2 ml = *reinterpret_cast<const float2 *>(a.part_ml + row * 2);
        const float4v op = *reinterpret_cast<const float4v *>(a.part_o + row * D + d4 * 4);
        const float m_new = fmaxf(m_all, ml.x);
        const float wa = exp2f(m_all - m_new), wb = exp2f(ml.x - m_new);  // a partial without visible tokens has l = 0
        l_all = l_all * wa + ml.y * wb;
        o = o * wa + op * wb;
        m_all = m_new;
    }
    const float inv = 1.f / l_all;
    const int qi = a.q_lo + n / G, hh = n % G;
    const long long orow = (long long)(q0 + qi) * a.num_q_heads + g * G + hh;
    const float2v lo = {o.x * inv, o.y * inv}, hi = {o.z * inv, o.w * inv};
    uint2 pk;
    pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
    pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
    *reinterpret_cast<uint2 *>(static_cast<__bf16 *>(a.out) + orow * D + d4 * 4) = pk;
    if (a.lse && d4 == 0) a.lse[orow] = (m_all + log2f(l_all)) * kLn2;
}

template <int G, int NB, bool FP8, bool TREE>
int32_t launch_stream(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1)
{
    // One wavefront per SIMD (the whole register file, a ring of NBUF tiles): two waves on a SIMD
    // do not share the memory pipeline fairly under saturation (the older one wins), which turns
    // into a long tail.
    constexpr bool QLDS = NB >= 4;
    constexpr int NBUF = NB <= 3 ? 4 : (NB == 5 && !FP8) ? 2 : 3;
    AttnArgs b = a;   // (the plan kernel has been enqueued by the caller)
    b.chain = kChainMerge<NB> ? 1 : 0;
    // When a profile is being taken the two events are attached to the dispatch itself, so that
    // their difference is the kernel's own duration on this stream (what a kernel trace shows).
    hipExtLaunchKernelGGL((attn_stream_kernel<G, NB, FP8, NBUF, QLDS, TREE>), dim3((unsigned)(b.launch_waves / kWavesPerWg)),
                          dim3(64 * kWavesPerWg), 0, stream, ev0, ev1, 0, b, b.tile_addr, b.wave_desc, b.tile_prefix,
                          b.kv_len, b.q_indptr, b.k_scale, b.v_scale);
    SS_HIP_CHECK(hipGetLastError(), "launch attn_stream_kernel");
    hipLaunchKernelGGL(attn_merge_kernel<G>, dim3((unsigned)a.batch * a.num_kv_heads * (a.rows_pad / kMergeRows)), dim3(256),
                       0, stream, b);
    SS_HIP_CHECK(hipGetLastError(), "launch attn_merge_kernel");
    return SS_OK;
}

template <int G, int NB>
int32_t launch_nb(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1)
{
    if (a.tree_mask) {
        if (a.kv_dtype == SS_FP8_E4M3) return launch_stream<G, NB, true, true>(a, stream, ev0, ev1);
        return launch_stream<G, NB, false, true>(a, stream, ev0, ev1);
    }
    if (a.kv_dtype == SS_FP8_E4M3) return launch_stream<G, NB, true, false>(a, stream, ev0, ev1);
    return launch_stream<G, NB, false, false>(a, stream, ev0, ev1);
}

template <int G>
int32_t launch_for_group(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1)
{
    constexpr int NBMAX = (SS_OUT_WIDTH * G + 15) / 16 < kMaxRowBlocks ? (SS_OUT_WIDTH * G + 15) / 16 : kMaxRowBlocks;
    const int nb = (a.q_win * G + 15) / 16;   // row blocks of one pass's window
    if constexpr (NBMAX >= 5) if (nb == 5) return launch_nb<G, 5>(a, stream, ev0, ev1);
    if constexpr (NBMAX >= 4) if (nb == 4) return launch_nb<G, 4>(a, stream, ev0, ev1);
    if constexpr (NBMAX >= 3) if (nb == 3) return launch_nb<G, 3>(a, stream, ev0, ev1);
    if constexpr (NBMAX >= 2) if (nb == 2) return launch_nb<G, 2>(a, stream, ev0, ev1);
    return launch_nb<G, 1>(a, stream, ev0, ev1);
}

}  // namespace
}  // namespace ss
