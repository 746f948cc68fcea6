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
// Roles inside a workgroup.  Eight wavefronts stream weights and multiply: each keeps a ring of ten 1 KiB chunks
// in flight, copied from global memory straight into LDS (no registers, so the ring position can be a run-time
// value and the loop stays small), and requests a new chunk for every chunk it multiplies, across stage
// boundaries.  Loads return in issue order, so a wavefront with weight requests in flight cannot also poll.  Four auxiliary
// wavefronts, which never touch the weights, fetch the stage's activation (polling the records of the stage
// before, or reading a caller tensor), run Eq.2 (Section 4.1) on it into LDS in MFMA operand order, and after the
// multiply add up the wavefronts' partial sums, dequantize per output channel (Section 4.4) and store.
//
// Every wait is bounded (a fixed number of polls, some tens of milliseconds): on a time-out a workgroup raises a sticky flag in the workspace and all
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
constexpr int kRing = 10;                            // 1 KiB weight chunks a streaming wavefront keeps in flight
constexpr int kHold = 24;                            // chunks a streaming lane moves on into registers before the
                                                     // activation is there (16 bytes each)
constexpr int kTG = 6;                               // channel tiles per workgroup and round
constexpr int kRows = 4;                             // token rows staged (M <= 4)
constexpr int kMaxKT = 128;                          // K <= 16384: 128 chunks x 512 B of codes in LDS
constexpr int kPB = 8;                               // 16-byte pieces a lane fetches per batch
constexpr int kMaxPolls = 100000;                    // polls before a wait gives up: each takes a trip to memory
                                                     // and back (0.3 us or more), so this is 30 ms at least
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
constexpr size_t kRingBytes = (size_t)kSWaves * kRing * 1024;         // 80 KiB: the weight chunks in flight
constexpr size_t kPartBytes = (size_t)kTG * kSWaves * 4 * 16 * 4;     // 12 KiB
constexpr size_t kLdsBytes = kXqBytes + kRingBytes + kPartBytes + 64;
static_assert(kLdsBytes <= 160 * 1024, "LDS of one compute unit");

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
    int nw;                                 // streaming wavefronts that own a K slice: ceil(KT / cpw)
    int tiles_base, tiles_rem;              // workgroup b serves tiles_base + (b < tiles_rem) tiles of the stage
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
// Weight pointers are typed as global memory: a pointer that comes out of a table has no known address space, and
// loads through it would be flat loads, which count as LDS traffic too and defeat the exact wait counts.
typedef const agq_u4 __attribute__((address_space(1))) *WeightPtr;

struct Cursor {
    int s, r, j, c;          // stage, round, tile slot of the round, chunk inside the wavefront's K slice
    int nj, nch;             // tiles of this workgroup in the round; chunks of this wavefront per tile
    // the stage's description, fetched once per stage (one round of scalar loads; fetching per tile would put two
    // dependent trips to memory in front of every fourth chunk)
    int KT, cpw, rounds, mine, t1, t2, t3;   // mine: tiles of this workgroup in the stage
    uint64_t blob0, blob1, blob2, blob3;   // addresses of the projections' blobs (integers: selected with scalar moves)
    WeightPtr base;          // first chunk of the slice in the current tile
    WeightPtr ptr;           // next chunk to request
    int left, step;          // chunks left in the current tile; 64 (16-byte units per chunk), 0 past the end
};

__device__ __forceinline__ void enter_stage(Cursor &k, StagePtr table, int b) {
    StagePtr st = table + k.s;
    k.KT = st->KT;
    k.cpw = st->cpw;
    k.rounds = st->rounds;
    k.mine = st->tiles_base + (b < st->tiles_rem ? 1 : 0);
    k.t1 = st->tile_start[1];
    k.t2 = st->tile_start[2];
    k.t3 = st->tile_start[3];
    k.blob0 = (uint64_t)st->blob[0];
    k.blob1 = (uint64_t)st->blob[1];
    k.blob2 = (uint64_t)st->blob[2];
    k.blob3 = (uint64_t)st->blob[3];
}

__device__ __forceinline__ void enter_round(Cursor &k, int b, int G, int wave) {
    k.nch = max(0, min(k.cpw, k.KT - wave * k.cpw));
    k.nj = k.nch > 0 ? max(0, min(kTG, k.mine - k.r * kTG)) : 0;
    k.j = 0;
    k.c = 0;
}

__device__ __forceinline__ void enter_tile(Cursor &k, int b, int G, int wave) {
    const int tile = b + (k.r * kTG + k.j) * G;
    const int pj = (tile >= k.t1) + (tile >= k.t2) + (tile >= k.t3);
    const int nt = tile - ((k.t1 & -(int)(pj == 1)) | (k.t2 & -(int)(pj == 2)) | (k.t3 & -(int)(pj == 3)));
    // picked with masks rather than a conditional: the compiler turns a conditional between struct fields into a
    // choice between their addresses, which pins the whole cursor to (scratch) memory
    const uint64_t blob = (k.blob0 & (0 - (uint64_t)(pj == 0))) | (k.blob1 & (0 - (uint64_t)(pj == 1))) |
                          (k.blob2 & (0 - (uint64_t)(pj == 2))) | (k.blob3 & (0 - (uint64_t)(pj == 3)));
    k.base = (WeightPtr)(blob + (uint64_t)((int64_t)nt * k.KT + wave * k.cpw) * 1024u);
}

// Moves the request cursor onto the next tile that has chunks for this wavefront (the next round's or stage's when
// the round is used up).  Past the end of the chain the cursor stays on a valid address and stops advancing, so
// that every multiplied chunk is still followed by exactly one request and the count of outstanding copies is
// constant.
__device__ __forceinline__ void issue_refill(Cursor &k, StagePtr table, int n_stages, int b, int G, int wave) {
    ++k.j;
    while (k.j >= k.nj) {
        if (++k.r >= k.rounds) {
            k.r = 0;
            if (++k.s >= n_stages) {
                k.s = n_stages;
                k.step = 0;              // the end: keep re-requesting the last tile's first chunk
                k.left = 0x7fffffff;
                k.ptr = k.base;
                return;
            }
            enter_stage(k, table, b);
        }
        enter_round(k, b, G, wave);
    }
    enter_tile(k, b, G, wave);
    k.ptr = k.base;
    k.left = k.nch;
}

// address (without the lane) of the next chunk to request
__device__ __forceinline__ WeightPtr issue_next(Cursor &k, StagePtr table, int n_stages, int b, int G, int wave) {
    if (k.left == 0) issue_refill(k, table, n_stages, b, G, wave);
    const WeightPtr p = k.ptr;
    k.ptr += k.step;
    --k.left;
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

// Direct global-to-LDS copy of 16 bytes per lane into a slot the wavefront has just read: the reads must have
// returned before the copy may overwrite the slot.
__device__ __forceinline__ void lds_dma16_after_reads(const void *gsrc, uint32_t lds_addr) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gsrc), "s"(lds_addr)
                 : "memory", "m0");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for every outstanding global
// load of the wavefront, i.e. for the whole weight stream in flight, at every round.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The workgroup's give-up flag in LDS, read as a wave-uniform value (a branch on the raw value would count as
// divergent).  The pointer is typed as LDS: through a generic pointer the read becomes a flat load, which waits
// for the wavefront's global loads as well.
typedef volatile int __attribute__((address_space(3))) *DeadPtr;
__device__ __forceinline__ bool is_dead(DeadPtr dead) { return __builtin_amdgcn_readfirstlane(*dead) != 0; }

// Marks the workspace as timed out (sticky) and notes, for whoever debugs it, the first workgroup that gave up
// without having seen the mark: word 8 = 1 + (workgroup << 16 | stage << 2 | which wait).
__device__ __forceinline__ void raise_abort(uint32_t *hdr, int b, int s, int kind) {
    if (__hip_atomic_load(&hdr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
        uint32_t expected = 0;
        __hip_atomic_compare_exchange_strong(&hdr[8], &expected, 1u + ((uint32_t)b << 16 | (uint32_t)s << 2 | (uint32_t)kind),
                                             __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __hip_atomic_store(&hdr[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A batch of record pairs (16 bytes each) with device-scope loads that bypass L2.  The two 8-byte halves of a pair
// are each written by one store; nothing is assumed about the 16 bytes as a whole, every record is checked by its own
// epoch.  The loads and the wait for them are ONE statement: the compiler takes an asm statement's outputs as ready
// when it ends, so a separate wait would leave it free to copy the registers before the data is in them.
__device__ __forceinline__ void poll_records(agq_u4 (&v)[kPB], const unsigned long long *const (&p)[kPB]) {
    static_assert(kPB == 8, "one operand pair per batch entry");
    asm volatile(
        "global_load_dwordx4 %0, %8, off sc1\n\t"
        "global_load_dwordx4 %1, %9, off sc1\n\t"
        "global_load_dwordx4 %2, %10, off sc1\n\t"
        "global_load_dwordx4 %3, %11, off sc1\n\t"
        "global_load_dwordx4 %4, %12, off sc1\n\t"
        "global_load_dwordx4 %5, %13, off sc1\n\t"
        "global_load_dwordx4 %6, %14, off sc1\n\t"
        "global_load_dwordx4 %7, %15, off sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
        : "v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3]), "v"(p[4]), "v"(p[5]), "v"(p[6]), "v"(p[7])
        : "memory");
}

// What the auxiliary wavefronts need of a stage, held in (scalar) registers: fetched for stage s + 1 while stage s
// is being multiplied.
struct AuxStage {
    const void *x;
    int64_t ldx;
    int t1, t2, t3, KT, nw, rounds, tiles_total, row_entries, src_off_entries, src_row_entries, feeds_next, K;
    float scale_e;
    AgqQuant q;
};

__device__ __forceinline__ void load_aux(AuxStage &a, StagePtr st) {
    a.x = st->x;
    a.ldx = st->ldx;
    a.t1 = st->tile_start[1];
    a.t2 = st->tile_start[2];
    a.t3 = st->tile_start[3];
    a.KT = st->KT;
    a.nw = st->nw;
    a.rounds = st->rounds;
    a.tiles_total = st->tiles_total;
    a.row_entries = st->row_entries;
    a.src_off_entries = st->src_off_entries;
    a.src_row_entries = st->src_row_entries;
    a.feeds_next = st->feeds_next;
    a.K = st->K;
    a.scale_e = st->scale_e;
    a.q.scale = st->q.scale;
    a.q.lo = st->q.lo;
    a.q.hi = st->q.hi;
    a.q.zp = st->q.zp;
    a.q.h_scale2 = st->q.h_scale2;
    a.q.h_lo2 = st->q.h_lo2;
    a.q.h_hi2 = st->q.h_hi2;
    a.q.h_zp2 = st->q.h_zp2;
}

// What one auxiliary lane stores in a round: channel pair cp of row m of the round's t-th tile.  Everything that
// depends on the lane's projection is fetched with vector loads (sixteen more scalar registers per stage
// description would spill); for the first round of a stage this runs one stage ahead, while the other wavefronts
// multiply, so that its two dependent trips to memory are off the chain between stages.
struct LaneOut {
    bool store;
    uint32_t sw2;        // the two channels' fp16 scales
    int32_t *pacc;       // &acc[m][n], or nullptr
    __half *py;          // &y[m][n]
    int rec_at;          // record index inside a row of the stage's records
};
typedef const ChainStage __attribute__((address_space(1))) *StageGlobalPtr;

__device__ __forceinline__ LaneOut lane_out(StageGlobalPtr table_g, int s, int r, int t1, int t2, int t3, int tiles_total,
                                            int b, int G, int t, int m, int cp, int M) {
    const int tile = b + (r * kTG + t) * G;
    const bool live = t < kTG && m < M && tile < tiles_total;
    const int tl = live ? tile : 0;
    const int pj = (tl >= t1) + (tl >= t2) + (tl >= t3);
    const int nt = tl - (pj == 0 ? 0 : (pj == 1 ? t1 : (pj == 2 ? t2 : t3)));
    const int n = nt * 16 + 2 * cp;
    StageGlobalPtr stg = table_g + s;
    const int pN = stg->N[pj], ldy = stg->ldy[pj], n_off = stg->n_off[pj];
    const __half *psw = stg->sw[pj];
    __half *y = stg->y[pj];
    int32_t *acc = stg->acc[pj];
    LaneOut o;
    o.store = live && n < pN;
    o.sw2 = 0;
    if (o.store) o.sw2 = *(const uint32_t __attribute__((address_space(1))) *)(psw + n);
    o.pacc = acc ? acc + (int64_t)m * pN + n : nullptr;
    o.py = y + (int64_t)m * ldy + n;
    o.rec_at = (n_off + n) >> 1;
    return o;
}

__global__ __launch_bounds__(kThreads) void gemm_chain_kernel(unsigned char *ws) {
    extern __shared__ __align__(16) unsigned char smem[];
    agq_u4 *xq = reinterpret_cast<agq_u4 *>(smem);
    int *part = reinterpret_cast<int *>(smem + kXqBytes + kRingBytes);
    DeadPtr dead = (DeadPtr)(smem + kXqBytes + kRingBytes + kPartBytes);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.x, G = gridDim.x;
    uint32_t *hdr = reinterpret_cast<uint32_t *>(ws);
    const ChainHeader *head = reinterpret_cast<const ChainHeader *>(ws);
    uint32_t *flags = reinterpret_cast<uint32_t *>(ws + kHdrBytes);
    StagePtr table = (StagePtr)(ws + kTableOff);
    StageGlobalPtr table_g = (StageGlobalPtr)(ws + kTableOff);   // the same, for vector loads
    const int n_stages = head->n_stages, M = head->M;
    const size_t ll_parity_entries = head->parity_entries;
    unsigned long long *ll = reinterpret_cast<unsigned long long *>(ws + head->ll_off);
    const uint32_t gen = hdr[0];
    if (__hip_atomic_load(&hdr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;   // an earlier launch timed out
    if (threadIdx.x == 0) {
        dead[0] = 0;
        dead[1] = 0;   // second word: the auxiliary wavefronts' "a workgroup is two stages behind" note
    }
    __syncthreads();

    if (wave < kSWaves) {
        // ------------------------------------------------------------ weight stream and multiply
        Cursor ic;
        ic.s = ic.r = 0;
        ic.step = 64;
        ic.left = 0;
        ic.base = (WeightPtr)table->blob[0];
        enter_stage(ic, table, b);
        enter_round(ic, b, G, wave);
        ic.j = -1;                                         // the first request moves onto the first tile
        // the multiply side walks the same sequence kRing chunks behind; it needs the counts only
        int cs = 0, cr = 0, c_rounds = ic.rounds, c_nj = ic.nj, c_nch = ic.nch, c_cpw = ic.cpw;
        int c_KT = ic.KT, c_mine = ic.mine;
        const uint32_t ring0 = __builtin_amdgcn_readfirstlane(
                                   (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) unsigned char *)smem) +
                               (uint32_t)kXqBytes + (uint32_t)wave * (kRing * 1024);
        const agq_u4 *ring = reinterpret_cast<const agq_u4 *>(smem + kXqBytes) + (size_t)wave * (kRing * 64) + lane;
        for (int i = 0; i < kRing; ++i)
            lds_dma16((const void *)(issue_next(ic, table, n_stages, b, G, wave) + lane), ring0 + (uint32_t)i * 1024u);
        const int ag = lane >> 4, srow = (lane & 15) & (kRows - 1);
        int slot = 0;                                      // ring position of the oldest chunk in flight
        // Chunks that have landed are moved on into registers while the wavefront waits for the stage's activation,
        // and their ring slots are refilled at once: the stream keeps running through the handoff between stages
        // instead of stopping when the ring is full.  (A register array needs compile-time indices, hence the
        // unrolled loops with a run-time count.)
        agq_u4 held[kHold];
        for (;;) {
            const int units = c_nj * c_nch;                // this wavefront's chunks in the round
            const int n_held = min(units, kHold);
#pragma unroll
            for (int i = 0; i < kHold; ++i) {
                if (i < n_held) {
                    // copies land in issue order: with kRing - 1 still outstanding the oldest is there
                    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kRing - 1) : "memory");
                    held[i] = ring[slot * 64];
                    lds_dma16_after_reads((const void *)(issue_next(ic, table, n_stages, b, G, wave) + lane),
                                          ring0 + (uint32_t)slot * 1024u);
                    slot = slot + 1 == kRing ? 0 : slot + 1;
                }
            }
            lds_barrier();                                 // B1: the stage's codes are in LDS, the partial sums consumed
            if (is_dead(dead)) return;
            int j = 0, c = 0;
            agq_v4i acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
            auto multiply = [&](const agq_u4 wv) {
                const int kc = wave * c_cpw + c;
                const agq_v4i a0 = __builtin_bit_cast(agq_v4i, xq[(kc * 8 + ag) * kRows + srow]);
                const agq_v4i a1 = __builtin_bit_cast(agq_v4i, xq[(kc * 8 + 4 + ag) * kRows + srow]);
                const agq_v4i b0 = __builtin_bit_cast(agq_v4i, (wv << 4) & 0xF0F0F0F0u);
                const agq_v4i b1 = __builtin_bit_cast(agq_v4i, wv & 0xF0F0F0F0u);
                acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1, acc1, 0, 0, 0);
                if (++c == c_nch) {                        // the tile's K slice is done
                    if (lane < 16) {                       // rows 0..3 of the 16 x 16 result live in lanes 0..15
#pragma unroll
                        for (int q = 0; q < 4; ++q) part[((j * kSWaves + wave) * 4 + q) * 16 + lane] = acc0[q] + acc1[q];
                    }
                    acc0 = agq_v4i{0, 0, 0, 0};
                    acc1 = agq_v4i{0, 0, 0, 0};
                    c = 0;
                    ++j;
                }
            };
#pragma unroll
            for (int i = 0; i < kHold; ++i)
                if (i < n_held) multiply(held[i]);
            for (int u = n_held; u < units; ++u) {         // a round with more chunks than registers: from the ring
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kRing - 1) : "memory");
                const agq_u4 wv = ring[slot * 64];
                lds_dma16_after_reads((const void *)(issue_next(ic, table, n_stages, b, G, wave) + lane),
                                      ring0 + (uint32_t)slot * 1024u);
                slot = slot + 1 == kRing ? 0 : slot + 1;
                multiply(wv);
            }
            lds_barrier();                                 // B2: this round's partial sums are in LDS
            if (is_dead(dead)) return;
            if (++cr >= c_rounds) {
                cr = 0;
                if (++cs >= n_stages) break;
                StagePtr st = table + cs;
                c_rounds = st->rounds;
                c_cpw = st->cpw;
                c_KT = st->KT;
                c_mine = st->tiles_base + (b < st->tiles_rem ? 1 : 0);
            }
            c_nch = max(0, min(c_cpw, c_KT - wave * c_cpw));
            c_nj = c_nch > 0 ? max(0, min(kTG, c_mine - cr * kTG)) : 0;
        }
        // the requests past the end of the chain still point into LDS: let them land before the wavefront ends
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    // ---------------------------------------------------------------- auxiliary wavefronts
    const int al = threadIdx.x - kSWaves * 64;         // 0..255
    // This lane's output of a round: channel pair cp of row m of the round's t-th tile.
    const int t = al >> 5, m = (al >> 3) & 3, cp = al & 7;
    AuxStage cur, nxt;
    load_aux(cur, table);
    nxt = cur;
    LaneOut lo = lane_out(table_g, 0, 0, cur.t1, cur.t2, cur.t3, cur.tiles_total, b, G, t, m, cp, M);
    LaneOut lo_next = lo;
    for (int s = 0; s < n_stages; ++s) {
        const int KT = cur.KT, K4 = cur.K >> 2;        // K4: 4-value pieces per row
        // The records of this stage will overwrite those of stage s - 2: every workgroup must have finished reading
        // them, which it has once it holds the input of stage s - 1 and says so in its progress word.  The words are
        // requested now, together with the first records, so the look costs no trip of its own.
        const bool credit_needed = cur.feeds_next && s >= 2;
        uint32_t early_word = 0;                       // looked at only after the first records have arrived
        if (credit_needed) early_word = __hip_atomic_load(&flags[min(al, G - 1)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // ---- the stage's activation -> codes in LDS (operand order [chunk][k half, k group][row] x 16 bytes)
        {
            const uint32_t want = gen + (uint32_t)s;   // epoch of the stage before
            const unsigned long long *src =
                ll + (size_t)((s + 1) & 1) * ll_parity_entries + cur.src_off_entries;   // parity of stage s - 1
            // A piece = four consecutive values of one row (two records).  Lane al takes the pieces al, al + 256, ...
            // of every row; a batch holds kPB of them, walking the rows in order (no division anywhere).
            const int per_row = (K4 + kALanes - 1) >> 8;   // pieces per lane and row
            static_assert(kALanes == 256, "the shift above");
            const int total = M * per_row;
            bool failed = false;
            int bm = 0, bi = 0;                        // row and in-row index of the batch's first piece
            for (int j0 = 0; j0 < total && !failed; j0 += kPB) {
                uint32_t d0[kPB], d1[kPB];
                int pm[kPB], pc4[kPB];                 // row and piece-in-row of every batch entry (pc4 < 0: none)
                {
                    int mm = bm, ii = bi;
#pragma unroll
                    for (int i = 0; i < kPB; ++i) {
                        const int c4 = ii * kALanes + al;
                        pm[i] = mm;
                        pc4[i] = (mm < M && c4 < K4) ? c4 : -1;
                        if (++ii == per_row) {
                            ii = 0;
                            ++mm;
                        }
                    }
                    bm = mm;
                    bi = ii;
                }
                if (cur.x != nullptr) {
#pragma unroll
                    for (int i = 0; i < kPB; ++i) {
                        const int mm = min(pm[i], M - 1), c4 = max(pc4[i], 0);
                        const uint2 v = *reinterpret_cast<const uint2 *>(reinterpret_cast<const __half *>(cur.x) +
                                                                          (int64_t)mm * cur.ldx + 4 * c4);
                        d0[i] = v.x;
                        d1[i] = v.y;
                    }
                } else {
                    const unsigned long long *p[kPB];
                    agq_u4 rec[kPB];                   // two records: (values, epoch, values, epoch)
#pragma unroll
                    for (int i = 0; i < kPB; ++i) {
                        const int mm = min(pm[i], M - 1), c4 = max(pc4[i], 0);
                        p[i] = src + (size_t)mm * cur.src_row_entries + 2 * c4;
                    }
                    for (int polls = 0;; ++polls) {
                        // the whole batch is asked for again until all of it carries the epoch (a record that has
                        // arrived stays: nothing overwrites it before every workgroup has read it)
                        poll_records(rec, p);
                        bool again = false;
#pragma unroll
                        for (int i = 0; i < kPB; ++i) again |= rec[i][1] != want || rec[i][3] != want;
                        if (__builtin_amdgcn_ballot_w64(again) == 0) break;
                        // give up after kMaxPolls, or (looked at every 64th poll) when another workgroup has
                        if (polls >= kMaxPolls || ((polls & 63) == 63 && __hip_atomic_load(&hdr[1], __ATOMIC_RELAXED,
                                                                                          __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                            failed = true;                                  // wave-uniform: the wavefront gives up as one
                            break;
                        }
                    }
#pragma unroll
                    for (int i = 0; i < kPB; ++i) {
                        d0[i] = rec[i][0];
                        d1[i] = rec[i][2];
                    }
                }
                if (failed) break;
#pragma unroll
                for (int i = 0; i < kPB; ++i) {
                    if (pc4[i] >= 0) {
                        const int k = 4 * pc4[i], kc = k >> 7, kk = k & 127;
                        const int piece = (kc * 8 + (kk >> 6) * 4 + ((kk >> 4) & 3)) * kRows + pm[i];
                        reinterpret_cast<uint32_t *>(xq)[piece * 4 + ((kk & 15) >> 2)] = quant4(d0[i], d1[i], cur.q);
                    }
                }
            }
            if (failed) {
                *dead = 1;
                raise_abort(hdr, b, s, 1);
            } else if (al == 0) {
                // progress: this workgroup no longer reads the records of stage s - 1
                __hip_atomic_store(&flags[b], gen + (uint32_t)s + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // any lane of any auxiliary wavefront behind -> all of them wait (through the LDS word next to `dead`); with
        // more workgroups than auxiliary lanes the early look does not cover all of them, so the full look always runs
        if (credit_needed && ((int)(early_word - (gen + (uint32_t)s)) < 0 || G > kALanes)) dead[1] = 1;
        const int rounds = cur.rounds;
        const int nw = cur.nw;                         // streaming wavefronts that own a K slice
        for (int r = 0; r < rounds; ++r) {
            // a second round of the same stage (more than kTG tiles per workgroup): set up here, in the chain
            if (r > 0) lo = lane_out(table_g, s, r, cur.t1, cur.t2, cur.t3, cur.tiles_total, b, G, t, m, cp, M);
            lds_barrier();                           // B1
            if (is_dead(dead)) return;
            const bool credit_pending = r == 0 && __builtin_amdgcn_readfirstlane(dead[1]) != 0;
            // While the other wavefronts multiply: fetch the description of the next stage (its scalar loads would
            // otherwise sit in the chain between two stages), and make sure this stage's records may be written.
            if (r + 1 == rounds && s + 1 < n_stages) {
                load_aux(nxt, table + (s + 1));
                // and what this lane will store in that stage's first round (two dependent trips to memory)
                lo_next = lane_out(table_g, s + 1, 0, nxt.t1, nxt.t2, nxt.t3, nxt.tiles_total, b, G, t, m, cp, M);
            }
            if (credit_pending && r == 0) {
                // (rare: the early look above found a workgroup two stages behind) wait here, off the critical path
                const uint32_t need = gen + (uint32_t)s;
                for (int polls = 0;; ++polls) {
                    bool behind = false;
                    for (int i = al; i < G; i += kALanes)
                        behind |= (int)(__hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - need) < 0;
                    if (__builtin_amdgcn_ballot_w64(behind) == 0) break;
                    if (polls >= kMaxPolls || ((polls & 63) == 63 && __hip_atomic_load(&hdr[1], __ATOMIC_RELAXED,
                                                                                      __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                        *dead = 1;
                        raise_abort(hdr, b, s, 2);
                        break;
                    }
                }
            }
            // everything the store needs, ready before the partial sums are
            unsigned long long *const dst = ll + (size_t)(s & 1) * ll_parity_entries + (size_t)m * cur.row_entries + lo.rec_at;
            const __half2 sc = __builtin_bit_cast(__half2, lo.sw2);
            const float g0 = cur.scale_e * __low2float(sc), g1 = cur.scale_e * __high2float(sc);
            lds_barrier();                           // B2
            if (is_dead(dead)) return;
            if (credit_pending && al == 0) dead[1] = 0;   // every auxiliary wavefront has read it (before B2)
            if (lo.store) {
                int s0 = 0, s1 = 0;
                for (int wv = 0; wv < nw; ++wv) {
                    const int2 v = *reinterpret_cast<const int2 *>(&part[((t * kSWaves + wv) * 4 + m) * 16 + 2 * cp]);
                    s0 += v.x;
                    s1 += v.y;
                }
                const int v0 = s0 >> AGQ_W_SHIFT, v1 = s1 >> AGQ_W_SHIFT;   // exact: every term carries the factor
                const __half y0 = agq_dequant(v0, g0), y1 = agq_dequant(v1, g1);
                const uint32_t ybits = (uint32_t)__half_as_ushort(y0) | ((uint32_t)__half_as_ushort(y1) << 16);
                if (cur.feeds_next)      // first: this is what the other compute units wait for
                    __hip_atomic_store(dst, ((unsigned long long)(gen + (uint32_t)s + 1u) << 32) | ybits, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                *reinterpret_cast<uint32_t *>(lo.py) = ybits;
                if (lo.pacc) *reinterpret_cast<int2 *>(lo.pacc) = make_int2(v0, v1);
            }
        }
        cur = nxt;
        lo = lo_next;
    }
    // The next launch starts a fresh range of epochs.  The base may only move once every workgroup has read it: each
    // publishes a progress word right after its first stage's input, so workgroup 0 waits for all of those.
    if (b == 0 && al < 64) {
        const uint32_t need = gen + 1u;
        bool ok = true;
        for (int polls = 0;; ++polls) {
            bool behind = false;
            for (int i = al; i < G; i += 64)
                behind |= (int)(__hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - need) < 0;
            if (__builtin_amdgcn_ballot_w64(behind) == 0) break;
            if (polls >= kMaxPolls || ((polls & 63) == 63 &&
                                       __hip_atomic_load(&hdr[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                ok = false;
                break;
            }
        }
        if (al == 0) {
            if (ok) hdr[0] = gen + (uint32_t)n_stages + 1u;
            else raise_abort(hdr, b, n_stages, 3);
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
        d.tiles_base = tiles / G;
        d.tiles_rem = tiles % G;
        d.nw = (d.KT + d.cpw - 1) / d.cpw;
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
