// A chain of quantized linear layers for a few tokens in ONE launch (the decode regime).
//
// With one launch per layer the HBM stream stops at every kernel boundary: requests start only after the launch
// and the last bytes must arrive before the next launch begins, which on this chip caps a pass of 8-45 MB reads
// at under 60 % of the HBM rate whatever the kernel does.  Here one persistent workgroup per compute unit walks
// through all stages.  The 4-bit weights of a stage do not depend on any activation, so each workgroup requests
// the weights of stage s+1 as soon as it has multiplied stage s; they are in flight while the outputs of stage s
// travel to the other workgroups.
//
// Handoff between stages.  The L2 caches of the chip's dies are not coherent with each other inside a launch, and
// invalidating them costs tens of microseconds, so a stage's outputs reach their readers through memory in a
// self-certifying form: every 8-byte record holds two fp16 values and the epoch (launch generation + stage) it
// was written in, stored and polled with device-scope accesses that bypass L2.  A record whose epoch matches is
// by construction the value of this stage; no flag, no fence and no ordering between stores is needed, and a
// reader waits exactly for the records it multiplies.  The plain fp16 output tensor is written as well.
//
// Roles inside a workgroup.  Eight wavefronts stream weights (registers only) and multiply; loads return in
// issue order, so a wavefront with megabytes of weight requests in flight cannot also poll.  Four auxiliary
// wavefronts, which never touch the weights, fetch the stage's activation (polling the records of the stage
// before, or reading a caller tensor), run Eq.2 (Section 4.1) on it into LDS in MFMA operand order, and after the
// multiply add up the wavefronts' partial sums, dequantize per output channel (Section 4.4) and store.
//
// Every wait is bounded (20 ms): on a time-out a workgroup raises a sticky flag in the workspace and all
// workgroups leave; later launches on that workspace return at once until it is prepared again.
#include <mutex>
#include <vector>

#include "../../include/agq.h"
#include "agq_device.h"
#include "agq_internal.h"

AgqQuant agq_make_quant_signed(int bits, int e, int zp);

namespace {

constexpr int kSWaves = 8;                           // weight-streaming wavefronts
constexpr int kAWaves = 4;                           // auxiliary wavefronts
constexpr int kThreads = (kSWaves + kAWaves) * 64;   // 768: three wavefronts per SIMD, up to 168 registers each
constexpr int kALanes = kAWaves * 64;
constexpr int kRing = 16;                            // 16-byte weight loads a streaming lane keeps in flight
constexpr int kTG = 8;                               // channel tiles per workgroup and round
constexpr int kRows = 4;                             // token rows staged (M <= 4)
constexpr int kMaxKT = 128;                          // K <= 16384: 128 chunks x 512 B of codes in LDS
constexpr int kPB = 8;                               // 16-byte pieces a lane fetches per batch
constexpr long long kWaitTicks = 2000000;            // 20 ms of the 100 MHz wall clock
constexpr int kMaxGrid = 1024;

// workspace layout (bytes)
struct ChainHeader {          // written by agq_gemm_chain_prepare; gen and abort change afterwards
    uint32_t gen;             // epoch base of the next launch
    uint32_t abort;           // sticky: a wait timed out
    int32_t n_stages, M;
    uint64_t ll_off;          // byte offset of the records
    uint64_t parity_entries;  // records per parity (M rows x half the widest stage)
};
constexpr size_t kHdrBytes = 256;
constexpr size_t kFlagBytes = kMaxGrid * 4;          // one progress word per workgroup
constexpr size_t kTableOff = kHdrBytes + kFlagBytes;

// LDS layout (bytes)
constexpr size_t kXqBytes = (size_t)kMaxKT * 8 * kRows * 16;          // 64 KiB
constexpr size_t kPartBytes = (size_t)kTG * kSWaves * 4 * 16 * 4;     // 16 KiB
constexpr size_t kLdsBytes = kXqBytes + kPartBytes + 64;

struct ChainStage {
    const void *x;              // caller's fp16 input, or nullptr: the records of the stage before
    int64_t ldx;
    const uint4 *blob[AGQ_MAX_PROJ];
    const __half *sw[AGQ_MAX_PROJ];
    __half *y[AGQ_MAX_PROJ];
    int32_t *acc[AGQ_MAX_PROJ];
    int N[AGQ_MAX_PROJ], ldy[AGQ_MAX_PROJ], n_off[AGQ_MAX_PROJ];
    int tile_start[AGQ_MAX_PROJ + 1];
    int count, KT, cpw, rounds, tiles_total, row_entries;   // cpw: chunks per streaming wavefront
    int src_off_entries, src_row_entries;   // x == nullptr: where the input sits inside a row of records
    int feeds_next;                         // a later stage reads this stage's output: write records
    float scale_e;
    int K;
    AgqQuant q;
};

typedef unsigned int agq_u4 __attribute__((ext_vector_type(4)));

// The stage table is read-only while the kernel runs.  Reading it through the constant address space makes every
// access a scalar load: a vector load here would queue behind the wavefront's weight stream (loads return in
// issue order) each time a cursor enters a new tile.
typedef const ChainStage __attribute__((address_space(4))) *StagePtr;

struct TileRef {
    int pj, nt;
};

// projection and tile index inside it of a stage's tile (any lane-varying tile id)
__device__ __forceinline__ TileRef tile_ref(StagePtr st, int tile) {
    const int t1 = st->tile_start[1], t2 = st->tile_start[2], t3 = st->tile_start[3];
    TileRef r;
    r.pj = (tile >= t1) + (tile >= t2) + (tile >= t3);
    r.nt = tile - (r.pj == 0 ? 0 : (r.pj == 1 ? t1 : (r.pj == 2 ? t2 : t3)));
    return r;
}

#define AGQ_PICK4(arr, pj) ((pj) == 0 ? (arr)[0] : ((pj) == 1 ? (arr)[1] : ((pj) == 2 ? (arr)[2] : (arr)[3])))

// The weight stream of one streaming wavefront: the 1 KiB chunks it multiplies, in the order it multiplies them
// (stage by stage, round by round, tile by tile, its own K slice of each tile front to back).  Two cursors walk
// this sequence, one for the requests and one, kRing chunks behind, for the multiply.  All fields are wave-uniform.
struct Cursor {
    int s, r, j, c;          // stage, round, tile slot of the round, chunk inside the wavefront's K slice
    int nj, nch;             // tiles of this workgroup in the round; chunks of this wavefront per tile
    int cpw, rounds;
    const agq_u4 *base;      // first chunk of the slice in the current tile
};

__device__ __forceinline__ void enter_round(Cursor &k, StagePtr table, int b, int G, int wave) {
    StagePtr st = table + k.s;
    const int cpw = st->cpw, KT = st->KT, tiles_total = st->tiles_total;
    k.cpw = cpw;
    k.rounds = st->rounds;
    k.nch = max(0, min(cpw, KT - wave * cpw));
    const int mine = b < tiles_total ? (tiles_total - b + G - 1) / G : 0;
    k.nj = k.nch > 0 ? max(0, min(kTG, mine - k.r * kTG)) : 0;
    k.j = 0;
    k.c = 0;
}

__device__ __forceinline__ void enter_tile(Cursor &k, StagePtr table, int b, int G, int wave) {
    StagePtr st = table + k.s;
    const TileRef tr = tile_ref(st, b + (k.r * kTG + k.j) * G);
    const uint4 *blob = AGQ_PICK4(st->blob, tr.pj);
    k.base = reinterpret_cast<const agq_u4 *>(blob) + ((int64_t)tr.nt * st->KT + wave * st->cpw) * 64;
}

// Address (without the lane) of the next chunk to request; past the end of the chain the last address again, so
// that every position of the ring issues exactly one load (the compiler then counts outstanding loads exactly).
__device__ __forceinline__ const agq_u4 *issue_next(Cursor &k, bool &done, const agq_u4 *&last, StagePtr table,
                                                    int n_stages, int b, int G, int wave) {
    while (!done && k.j >= k.nj) {
        if (++k.r >= k.rounds) {
            k.r = 0;
            if (++k.s >= n_stages) {
                done = true;
                break;
            }
        }
        enter_round(k, table, b, G, wave);
        if (k.nj > 0) enter_tile(k, table, b, G, wave);
    }
    if (done) return last;
    const agq_u4 *p = k.base + k.c * 64;
    last = p;
    if (++k.c == k.nch) {
        k.c = 0;
        if (++k.j < k.nj) enter_tile(k, table, b, G, wave);
    }
    return p;
}

// four fp16 values (two words) -> four codes of Eq.2 on the signed grid in one word, k ascending
__device__ __forceinline__ uint32_t quant4(uint32_t h01, uint32_t h23, const AgqQuant &q) {
    if (q.h_scale2 != 0) {
        const uint32_t t0 = agq_quant2h<false>(h01, q), t1 = agq_quant2h<false>(h23, q);
        return __builtin_amdgcn_perm(t1, t0, 0x06040200u);
    }
    const float2 f0 = __half22float2(__builtin_bit_cast(__half2, h01));
    const float2 f1 = __half22float2(__builtin_bit_cast(__half2, h23));
    return agq_pack4(agq_quant1(f0.x, q), agq_quant1(f0.y, q), agq_quant1(f1.x, q), agq_quant1(f1.y, q));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for every outstanding global
// load of the wavefront, i.e. for the whole weight stream in flight, at every round.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The workgroup's give-up flag in LDS, read as a wave-uniform value (a branch on the raw value would count as
// divergent).  The pointer is typed as LDS: through a generic pointer the read becomes a flat load, which waits
// for the wavefront's global loads as well.
typedef volatile int __attribute__((address_space(3))) *DeadPtr;
__device__ __forceinline__ bool is_dead(DeadPtr dead) { return __builtin_amdgcn_readfirstlane(*dead) != 0; }

__device__ __forceinline__ unsigned long long load_record(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(kThreads) void gemm_chain_kernel(unsigned char *ws) {
    extern __shared__ __align__(16) unsigned char smem[];
    agq_u4 *xq = reinterpret_cast<agq_u4 *>(smem);
    int *part = reinterpret_cast<int *>(smem + kXqBytes);
    DeadPtr dead = (DeadPtr)(smem + kXqBytes + kPartBytes);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.x, G = gridDim.x;
    uint32_t *hdr = reinterpret_cast<uint32_t *>(ws);
    const ChainHeader *head = reinterpret_cast<const ChainHeader *>(ws);
    uint32_t *flags = reinterpret_cast<uint32_t *>(ws + kHdrBytes);
    StagePtr table = (StagePtr)(ws + kTableOff);
    const int n_stages = head->n_stages, M = head->M;
    const size_t ll_parity_entries = head->parity_entries;
    unsigned long long *ll = reinterpret_cast<unsigned long long *>(ws + head->ll_off);
    const uint32_t gen = hdr[0];
    if (__hip_atomic_load(&hdr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;   // an earlier launch timed out
    if (threadIdx.x == 0) *dead = 0;
    __syncthreads();

    if (wave < kSWaves) {
        // ------------------------------------------------------------ weight stream and multiply
        Cursor ic, cc;
        ic.s = ic.r = 0;
        enter_round(ic, table, b, G, wave);
        if (ic.nj > 0) enter_tile(ic, table, b, G, wave);
        cc = ic;
        bool issue_done = false;
        const agq_u4 *last = reinterpret_cast<const agq_u4 *>(table->blob[0]);
        agq_u4 w[kRing];
#pragma unroll
        for (int i = 0; i < kRing; ++i) w[i] = issue_next(ic, issue_done, last, table, n_stages, b, G, wave)[lane];
        const int ag = lane >> 4, srow = (lane & 15) & (kRows - 1);
        agq_v4i acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
        bool in_round = false;
        for (;;) {
#pragma unroll
            for (int i = 0; i < kRing; ++i) {
                // move the multiply cursor onto a chunk, passing the barriers of every round on the way:
                // B1 (the stage's codes are in LDS, the previous partial sums are consumed) before a round's first
                // chunk, B2 (this round's partial sums are in LDS) after its last; rounds without a chunk for this
                // wavefront pass both
                for (;;) {
                    if (!in_round) {
                        lds_barrier();
                        if (is_dead(dead)) return;
                        in_round = true;
                    }
                    if (cc.j < cc.nj) break;
                    lds_barrier();
                    if (is_dead(dead)) return;
                    in_round = false;
                    if (++cc.r >= cc.rounds) {
                        cc.r = 0;
                        if (++cc.s >= n_stages) return;
                    }
                    enter_round(cc, table, b, G, wave);
                }
                const int kc = wave * cc.cpw + cc.c;
                const agq_v4i a0 = __builtin_bit_cast(agq_v4i, xq[(kc * 8 + ag) * kRows + srow]);
                const agq_v4i a1 = __builtin_bit_cast(agq_v4i, xq[(kc * 8 + 4 + ag) * kRows + srow]);
                const agq_u4 wv = w[i];
                const agq_v4i b0 = __builtin_bit_cast(agq_v4i, (wv << 4) & 0xF0F0F0F0u);
                const agq_v4i b1 = __builtin_bit_cast(agq_v4i, wv & 0xF0F0F0F0u);
                acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1, acc1, 0, 0, 0);
                if (++cc.c == cc.nch) {
                    // the tile's K slice is done: rows 0..3 of the 16 x 16 result live in lanes 0..15
                    if (lane < 16) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) part[((cc.j * kSWaves + wave) * 4 + q) * 16 + lane] = acc0[q] + acc1[q];
                    }
                    acc0 = agq_v4i{0, 0, 0, 0};
                    acc1 = agq_v4i{0, 0, 0, 0};
                    cc.c = 0;
                    ++cc.j;
                }
                // the register is free again: request the chunk kRing places ahead (this stage's or a later one's)
                w[i] = issue_next(ic, issue_done, last, table, n_stages, b, G, wave)[lane];
            }
        }
    }

    // ---------------------------------------------------------------- auxiliary wavefronts
    const int al = threadIdx.x - kSWaves * 64;         // 0..255
    for (int s = 0; s < n_stages; ++s) {
        StagePtr st = table + s;
        AgqQuant stq;                                  // field by field: a struct copy cannot cross address spaces
        stq.scale = st->q.scale;
        stq.lo = st->q.lo;
        stq.hi = st->q.hi;
        stq.zp = st->q.zp;
        stq.h_scale2 = st->q.h_scale2;
        stq.h_lo2 = st->q.h_lo2;
        stq.h_hi2 = st->q.h_hi2;
        stq.h_zp2 = st->q.h_zp2;
        const int KT = st->KT, K4 = st->K >> 2;          // K4: 4-value pieces per row
        // ---- the stage's activation -> codes in LDS (operand order [chunk][k half, k group][row] x 16 bytes)
        {
            const int pieces = M * K4;
            const uint32_t want = gen + (uint32_t)s;   // epoch of the stage before
            const unsigned long long *src =
                ll + (size_t)((s + 1) & 1) * ll_parity_entries + st->src_off_entries;   // parity of stage s - 1
            bool failed = false;
            for (int j0 = 0; j0 < pieces && !failed; j0 += kALanes * kPB) {
                uint32_t d0[kPB], d1[kPB];
                if (st->x != nullptr) {
#pragma unroll
                    for (int i = 0; i < kPB; ++i) {
                        const int j = min(j0 + i * kALanes + al, pieces - 1);
                        const int m = j / K4, c4 = j - m * K4;
                        const uint2 v = *reinterpret_cast<const uint2 *>(reinterpret_cast<const __half *>(st->x) +
                                                                          (int64_t)m * st->ldx + 4 * c4);
                        d0[i] = v.x;
                        d1[i] = v.y;
                    }
                } else {
                    const unsigned long long *p[kPB];
                    unsigned long long r0[kPB], r1[kPB];
#pragma unroll
                    for (int i = 0; i < kPB; ++i) {
                        const int j = min(j0 + i * kALanes + al, pieces - 1);
                        const int m = j / K4, c4 = j - m * K4;
                        p[i] = src + (size_t)m * st->src_row_entries + 2 * c4;
                        r0[i] = load_record(p[i]);
                        r1[i] = load_record(p[i] + 1);
                    }
                    const long long t0 = wall_clock64();
                    for (;;) {
                        bool again = false;
#pragma unroll
                        for (int i = 0; i < kPB; ++i) {
                            if ((uint32_t)(r0[i] >> 32) != want) { r0[i] = load_record(p[i]); again = true; }
                            if ((uint32_t)(r1[i] >> 32) != want) { r1[i] = load_record(p[i] + 1); again = true; }
                        }
                        if (__builtin_amdgcn_ballot_w64(again) == 0) break;
                        const bool over = wall_clock64() - t0 > kWaitTicks ||
                                          __hip_atomic_load(&hdr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
                        if (__builtin_amdgcn_ballot_w64(over) != 0) {      // the wavefront gives up as one
                            failed = true;
                            break;
                        }
                    }
#pragma unroll
                    for (int i = 0; i < kPB; ++i) {
                        d0[i] = (uint32_t)r0[i];
                        d1[i] = (uint32_t)r1[i];
                    }
                }
                if (failed) break;
#pragma unroll
                for (int i = 0; i < kPB; ++i) {
                    const int j = j0 + i * kALanes + al;
                    if (j < pieces) {
                        const int m = j / K4, c4 = j - m * K4;
                        const int k = 4 * c4, kc = k >> 7, kk = k & 127;
                        const int piece = (kc * 8 + (kk >> 6) * 4 + ((kk >> 4) & 3)) * kRows + m;
                        reinterpret_cast<uint32_t *>(xq)[piece * 4 + ((kk & 15) >> 2)] = quant4(d0[i], d1[i], stq);
                    }
                }
            }
            if (failed) {
                *dead = 1;
                __hip_atomic_store(&hdr[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (al == 0) {
                // progress: this workgroup no longer reads the records of stage s - 1
                __hip_atomic_store(&flags[b], gen + (uint32_t)s + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        const int rounds = st->rounds;
        const int nw = min(kSWaves, (KT + st->cpw - 1) / st->cpw);   // streaming wavefronts that own a K slice
        for (int r = 0; r < rounds; ++r) {
            // this lane's output: channel pair cp of row m of the round's t-th tile
            const int t = al >> 5, m = (al >> 3) & 3, cp = al & 7;
            const int tile = b + (r * kTG + t) * G;
            const bool live = m < M && tile < st->tiles_total;
            const TileRef tr = tile_ref(st, live ? tile : 0);
            const int n = tr.nt * 16 + 2 * cp;
            const int pN = AGQ_PICK4(st->N, tr.pj);
            const bool store = live && n < pN;
            uint32_t sw2 = 0;
            if (store) sw2 = *reinterpret_cast<const uint32_t *>(AGQ_PICK4(st->sw, tr.pj) + n);   // scales of n and n + 1
            lds_barrier();                           // B1
            if (is_dead(dead)) return;
            if (st->feeds_next && s >= 2 && r == 0) {
                // The records of this stage overwrite those of stage s - 2: every workgroup must have finished
                // reading them (it has, once it holds the input of stage s - 1).  Checked here, off the critical
                // path, while the other wavefronts multiply.
                const uint32_t need = gen + (uint32_t)s;
                const long long t0 = wall_clock64();
                for (;;) {
                    bool behind = false;
                    for (int i = al; i < G; i += kALanes)
                        behind |= (int)(__hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - need) < 0;
                    if (__builtin_amdgcn_ballot_w64(behind) == 0) break;
                    const bool over = wall_clock64() - t0 > kWaitTicks ||
                                      __hip_atomic_load(&hdr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
                    if (__builtin_amdgcn_ballot_w64(over) != 0) {
                        *dead = 1;
                        __hip_atomic_store(&hdr[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                }
            }
            lds_barrier();                           // B2
            if (is_dead(dead)) return;
            if (store) {
                int s0 = 0, s1 = 0;
                for (int wv = 0; wv < nw; ++wv) {
                    const int2 v = *reinterpret_cast<const int2 *>(&part[((t * kSWaves + wv) * 4 + m) * 16 + 2 * cp]);
                    s0 += v.x;
                    s1 += v.y;
                }
                const int v0 = s0 >> AGQ_W_SHIFT, v1 = s1 >> AGQ_W_SHIFT;   // exact: every term carries the factor
                int32_t *pacc = AGQ_PICK4(st->acc, tr.pj);
                if (pacc) *reinterpret_cast<int2 *>(pacc + (int64_t)m * pN + n) = make_int2(v0, v1);
                const __half2 sc = __builtin_bit_cast(__half2, sw2);
                const __half y0 = agq_dequant(v0, st->scale_e * __low2float(sc));
                const __half y1 = agq_dequant(v1, st->scale_e * __high2float(sc));
                const uint32_t ybits = (uint32_t)__half_as_ushort(y0) | ((uint32_t)__half_as_ushort(y1) << 16);
                *reinterpret_cast<uint32_t *>(AGQ_PICK4(st->y, tr.pj) + (int64_t)m * AGQ_PICK4(st->ldy, tr.pj) + n) = ybits;
                if (st->feeds_next) {
                    unsigned long long *dst = ll + (size_t)(s & 1) * ll_parity_entries + (size_t)m * st->row_entries +
                                              ((AGQ_PICK4(st->n_off, tr.pj) + n) >> 1);
                    __hip_atomic_store(dst, ((unsigned long long)(gen + (uint32_t)s + 1u) << 32) | ybits, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
    // The next launch starts a fresh range of epochs.  The base may only move once every workgroup has read it: each
    // publishes a progress word right after its first stage's input, so workgroup 0 waits for all of those.
    if (b == 0 && al < 64) {
        const uint32_t need = gen + 1u;
        const long long t0 = wall_clock64();
        bool ok = true;
        for (;;) {
            bool behind = false;
            for (int i = al; i < G; i += 64)
                behind |= (int)(__hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - need) < 0;
            if (__builtin_amdgcn_ballot_w64(behind) == 0) break;
            const bool over = wall_clock64() - t0 > kWaitTicks ||
                              __hip_atomic_load(&hdr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
            if (__builtin_amdgcn_ballot_w64(over) != 0) {
                ok = false;
                break;
            }
        }
        if (al == 0) {
            if (ok) hdr[0] = gen + (uint32_t)n_stages + 1u;
            else __hip_atomic_store(&hdr[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int grid_of_device(int *out) {
    static int ncu_of[64] = {0};
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return AGQ_EHIP;
    int ncu = ncu_of[device];
    if (ncu == 0) {
        if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || ncu < 1) return AGQ_EHIP;
        ncu_of[device] = ncu;
    }
    *out = ncu < kMaxGrid ? ncu : kMaxGrid;
    return AGQ_OK;
}

// host-side checks of a chain; fills max_ntot (widest stage, all projections)
int check_chain(const agq_chain_stage *stages, int n_stages, int64_t M, int64_t *max_ntot) {
    if (!stages || n_stages < 1 || n_stages > AGQ_CHAIN_MAX_STAGES || M < 1 || M > AGQ_CHAIN_MAX_M) return AGQ_EINVAL;
    int64_t widest = 0;
    for (int s = 0; s < n_stages; ++s) {
        const agq_chain_stage &c = stages[s];
        if (c.K < 128 || c.K > (int64_t)kMaxKT * 128 || (c.K % 128) != 0) return AGQ_EINVAL;
        if ((c.bits != 4 && c.bits != 8) || c.e < AGQ_E_MIN || c.e > AGQ_E_MAX) return AGQ_EINVAL;
        if (c.count < 1 || c.count > AGQ_MAX_PROJ) return AGQ_EINVAL;
        int64_t ntot = 0;
        for (int p = 0; p < c.count; ++p) {
            const agq_proj &pr = c.projs[p];
            if (pr.N < 16 || pr.N > (1 << 24) || (pr.N % 16) != 0 || pr.ldy < pr.N || pr.ldy > ((int64_t)1 << 30) ||
                (pr.ldy % 2) != 0)
                return AGQ_EINVAL;
            if (!pr.w_packed || !pr.w_scale_f16 || !pr.y_f16) return AGQ_EINVAL;
            if (!aligned16(pr.w_packed) || !aligned16(pr.w_scale_f16) || !aligned16(pr.y_f16)) return AGQ_EINVAL;
            if (pr.acc_out && (reinterpret_cast<uintptr_t>(pr.acc_out) & 7) != 0) return AGQ_EINVAL;
            ntot += pr.N;
        }
        if (ntot > (1 << 24)) return AGQ_EINVAL;
        if (ntot > widest) widest = ntot;
        if (c.x_f16) {
            if (!aligned16(c.x_f16) || c.ldx < c.K || (c.ldx % 8) != 0) return AGQ_EINVAL;
        } else {
            if (s == 0) return AGQ_EINVAL;                               // the first stage reads a caller tensor
            const agq_chain_stage &prev = stages[s - 1];
            if (c.src_proj < 0 || c.src_proj >= prev.count || prev.projs[c.src_proj].N != c.K) return AGQ_EINVAL;
        }
    }
    *max_ntot = widest;
    return AGQ_OK;
}

size_t ll_offset(int n_stages) {
    const size_t end = kTableOff + (size_t)n_stages * sizeof(ChainStage);
    return (end + 255) / 256 * 256;
}

std::once_flag g_chain_once[64];
hipError_t g_chain_err[64];

int raise_chain_lds() {
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return AGQ_EHIP;
    std::call_once(g_chain_once[device], [device] {
        g_chain_err[device] = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_chain_kernel),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
    });
    return g_chain_err[device] == hipSuccess ? AGQ_OK : AGQ_EHIP;
}

}  // namespace

extern "C" size_t agq_gemm_chain_workspace_bytes(const agq_chain_stage *stages, int n_stages, int64_t M) {
    int64_t widest = 0;
    if (check_chain(stages, n_stages, M, &widest) != AGQ_OK) return 0;
    return ll_offset(n_stages) + (size_t)2 * (size_t)M * (size_t)(widest / 2) * 8;
}

extern "C" int agq_gemm_chain_prepare(const agq_chain_stage *stages, int n_stages, int64_t M, void *workspace,
                                      size_t workspace_bytes, void *stream) {
    int64_t widest = 0;
    const int st = check_chain(stages, n_stages, M, &widest);
    if (st != AGQ_OK) return st;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return AGQ_EINVAL;
    const size_t need = ll_offset(n_stages) + (size_t)2 * (size_t)M * (size_t)(widest / 2) * 8;
    if (workspace_bytes < need) return AGQ_ESIZE;
    int G = 0;
    if (grid_of_device(&G) != AGQ_OK || raise_chain_lds() != AGQ_OK) return AGQ_EHIP;

    std::vector<ChainStage> table((size_t)n_stages);
    for (int s = 0; s < n_stages; ++s) {
        const agq_chain_stage &c = stages[s];
        ChainStage &d = table[(size_t)s];
        d = ChainStage{};
        d.x = c.x_f16;
        d.ldx = c.ldx;
        d.K = (int)c.K;
        d.KT = (int)(c.K / 128);
        d.cpw = (d.KT + kSWaves - 1) / kSWaves;
        d.count = c.count;
        int tiles = 0, noff = 0;
        for (int p = 0; p < AGQ_MAX_PROJ; ++p) {
            const agq_proj &pr = c.projs[p < c.count ? p : c.count - 1];
            d.tile_start[p] = tiles;
            d.n_off[p] = noff;
            if (p < c.count) {
                tiles += (int)(pr.N / 16);
                noff += (int)pr.N;
            }
            d.blob[p] = (const uint4 *)pr.w_packed;
            d.sw[p] = (const __half *)pr.w_scale_f16;
            d.y[p] = (__half *)pr.y_f16;
            d.acc[p] = pr.acc_out;
            d.N[p] = (int)pr.N;
            d.ldy[p] = (int)pr.ldy;
        }
        for (int p = c.count; p <= AGQ_MAX_PROJ; ++p) d.tile_start[p] = tiles;
        d.tiles_total = tiles;
        d.row_entries = noff / 2;
        const int per_wg = (tiles + G - 1) / G;
        d.rounds = (per_wg + kTG - 1) / kTG;
        d.feeds_next = (s + 1 < n_stages && stages[s + 1].x_f16 == nullptr) ? 1 : 0;
        if (!c.x_f16) {
            const ChainStage &prev = table[(size_t)s - 1];
            d.src_row_entries = prev.row_entries;
            d.src_off_entries = prev.n_off[c.src_proj] / 2;
        }
        d.scale_e = ldexpf(1.0f, c.e);
        d.q = agq_make_quant_signed(c.bits, c.e, 0);
    }
    hipStream_t hs = (hipStream_t)stream;
    ChainHeader head = {};
    head.n_stages = n_stages;
    head.M = (int32_t)M;
    head.ll_off = ll_offset(n_stages);
    head.parity_entries = (uint64_t)M * (uint64_t)(widest / 2);
    // generation, time-out flag, progress words and every record start at zero (no epoch is ever zero)
    if (hipMemsetAsync(workspace, 0, need, hs) != hipSuccess) return AGQ_EHIP;
    if (hipMemcpyAsync(workspace, &head, sizeof(head), hipMemcpyHostToDevice, hs) != hipSuccess) return AGQ_EHIP;
    if (hipMemcpyAsync(static_cast<char *>(workspace) + kTableOff, table.data(), table.size() * sizeof(ChainStage),
                       hipMemcpyHostToDevice, hs) != hipSuccess)
        return AGQ_EHIP;
    return hipStreamSynchronize(hs) == hipSuccess ? AGQ_OK : AGQ_EHIP;   // the table is read from host memory
}

extern "C" int agq_gemm_chain_run(void *workspace, void *stream) {
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return AGQ_EINVAL;
    int G = 0;
    if (grid_of_device(&G) != AGQ_OK || raise_chain_lds() != AGQ_OK) return AGQ_EHIP;
    gemm_chain_kernel<<<(unsigned)G, kThreads, kLdsBytes, (hipStream_t)stream>>>(static_cast<unsigned char *>(workspace));
    return hipGetLastError() == hipSuccess ? AGQ_OK : AGQ_EHIP;
}

extern "C" int agq_gemm_chain_status(const void *workspace, void *stream) {
    if (!workspace) return AGQ_EINVAL;
    int32_t flag = 0;
    if (agq_read_i32(reinterpret_cast<const int32_t *>(workspace) + 1, &flag, 1, stream) != 0) return AGQ_EHIP;   // waits for the stream
    return flag == 0 ? AGQ_OK : AGQ_ETIMEOUT;
}
