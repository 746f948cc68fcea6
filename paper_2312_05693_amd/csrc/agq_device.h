// Device-side helpers shared by the agq kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

typedef int agq_v4i __attribute__((ext_vector_type(4)));

// Parameters of Eq.2 (Section 4.1) with s = 2^e, prepared on the host so that
// one fused multiply-add and one median do the whole quantizer:
//   r = x * 2^-e + MAGIC   rounds x/s to an integer (ties to even) because
//       floats in [2^23, 2^24) have a spacing of exactly 1 and MAGIC is even;
//   r = med3(r, MAGIC + lo - zp, MAGIC + hi - zp)   is the CLIP of round + zp;
//   the low byte of (bits(r) + zp) is the code in two's complement.
// The zero point is added after the rounding, as Eq.2 prints it: folding an odd
// zp into the fused add would flip the parity that decides ties.
struct AgqQuant {
    float scale;  // 2^-e
    float lo;     // MAGIC + lower grid bound - zp
    float hi;     // MAGIC + upper grid bound - zp
    int zp;
    // the same in packed fp16 pairs: 2^-e, 1536 + lower and 1536 + upper bound (minus zp);
    // h_scale2 == 0 when 2^-e is not a normal fp16 number.  h_zp2: the low byte
    // of zp in both halves, added to the bit patterns after rounding.
    uint32_t h_scale2, h_lo2, h_hi2, h_zp2;
};
#define AGQ_MAGIC 12582912.0f  // 1.5 * 2^23

__device__ __forceinline__ uint32_t agq_quant1(float x, const AgqQuant &q) {
    float r = fmaf(x, q.scale, AGQ_MAGIC);
    r = __builtin_amdgcn_fmed3f(r, q.lo, q.hi);
    return __float_as_uint(r);   // zero point not yet added
}

// low bytes of four 32-bit words -> one word, word 0 in byte 0
__device__ __forceinline__ uint32_t agq_pack4(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3) {
    uint32_t p01 = __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u);
    uint32_t p23 = __builtin_amdgcn_perm(b3, b2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(p23, p01, 0x05040100u);
}

// Eq.2 on the signed grid in packed fp16, eight values (four words) -> eight codes
// in two words, k ascending.  One fused multiply-add per pair, x * 2^-e + 1536 (1536 =
// 1.5 * 2^10; the product is exact, so this is a single rounding of the exact sum),
// rounds half-to-even to an integer k wherever the sum lands in [1024, 2048), i.e.
// for every k the grid can hold, and leaves k's two's complement in the low byte of
// the bit pattern 0x6600 + k; outside that interval the sum is rounded more coarsely
// or more finely, but monotonically, so the clamp to 1536 + (grid bounds) that follows
// gives the same code as clamping before the rounding would.  Three instructions per
// pair.  Requires q.h_scale2 != 0.  Built by agq_make_quant_signed: codes on the
// signed grid, zero point q.zp (may be negative).
typedef _Float16 agq_h2v __attribute__((ext_vector_type(2)));
template <bool ZP>
__device__ __forceinline__ uint32_t agq_quant2h(uint32_t two, const AgqQuant &q) {
    agq_h2v v = __builtin_elementwise_fma(__builtin_bit_cast(agq_h2v, two), __builtin_bit_cast(agq_h2v, q.h_scale2),
                                          agq_h2v{(_Float16)1536.0f, (_Float16)1536.0f});
    v = __builtin_elementwise_min(__builtin_elementwise_max(v, __builtin_bit_cast(agq_h2v, q.h_lo2)),
                                  __builtin_bit_cast(agq_h2v, q.h_hi2));
    // the zero point is added after the rounding (Eq.2 as printed); 0x66xx + zp stays
    // inside its half, so one 32-bit add serves both
    return ZP ? __builtin_bit_cast(uint32_t, v) + q.h_zp2 : __builtin_bit_cast(uint32_t, v);
}
template <bool ZP>
__device__ __forceinline__ uint2 agq_quant8h(uint32_t h0, uint32_t h1, uint32_t h2, uint32_t h3, const AgqQuant &q) {
    const uint32_t t0 = agq_quant2h<ZP>(h0, q), t1 = agq_quant2h<ZP>(h1, q), t2 = agq_quant2h<ZP>(h2, q),
                   t3 = agq_quant2h<ZP>(h3, q);
    return make_uint2(__builtin_amdgcn_perm(t1, t0, 0x06040200u), __builtin_amdgcn_perm(t3, t2, 0x06040200u));
}

// eight fp16 (one 16-byte load) -> eight codes in two words, k ascending.
// WITH_ZP = false is the signed grid (zp = 0) used by the GEMM prologues.
template <bool WITH_ZP = false>
__device__ __forceinline__ uint2 agq_quant8(const uint4 &h, const AgqQuant &q) {
    const __half2 *p = reinterpret_cast<const __half2 *>(&h);
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 f = __half22float2(p[i]);
        c[2 * i] = agq_quant1(f.x, q);
        c[2 * i + 1] = agq_quant1(f.y, q);
        if (WITH_ZP) {
            c[2 * i] += (uint32_t)q.zp;
            c[2 * i + 1] += (uint32_t)q.zp;
        }
    }
    uint2 out;
    out.x = agq_pack4(c[0], c[1], c[2], c[3]);
    out.y = agq_pack4(c[4], c[5], c[6], c[7]);
    return out;
}

// A word of the packed weight blob holds eight 4-bit weights: the low nibbles of
// its four bytes belong to MFMA step 0, the high nibbles to step 1.  Moving a
// nibble into the top half of its byte yields the weight times 16 as an int8
// (two's complement does the sign), so the int4 -> int8 widening costs three
// bit operations per eight weights and the factor 16 is shifted out of the
// int32 accumulator at the end.
#define AGQ_W_SHIFT 4
__device__ __forceinline__ void agq_unpack_w(const uint4 &p, agq_v4i &b0, agq_v4i &b1) {
    b0.x = (int)((p.x << 4) & 0xF0F0F0F0u); b1.x = (int)(p.x & 0xF0F0F0F0u);
    b0.y = (int)((p.y << 4) & 0xF0F0F0F0u); b1.y = (int)(p.y & 0xF0F0F0F0u);
    b0.z = (int)((p.z << 4) & 0xF0F0F0F0u); b1.z = (int)(p.z & 0xF0F0F0F0u);
    b0.w = (int)((p.w << 4) & 0xF0F0F0F0u); b1.w = (int)(p.w & 0xF0F0F0F0u);
}

// y = fp16( float(acc) * g ), g = 2^e * sw[n] prepared by the caller
__device__ __forceinline__ __half agq_dequant(int acc, float g) {
    return __float2half_rn((float)acc * g);
}

// Direct global-to-LDS copy: lane i's 16 bytes land at lds_chunk + 16 i (the LDS
// address is wave-uniform and travels in M0).  Issued as inline assembly on
// purpose: the compiler, seeing such a copy, drains every outstanding load
// (vmcnt(0)) before any later LDS read, which would cancel the prefetch distance;
// so a kernel that uses it waits for exactly the copies it needs with explicit
// s_waitcnt vmcnt(n) (loads, these included, return in order).
__device__ __forceinline__ void lds_dma16(const void *gsrc, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gsrc), "s"(lds_addr)
                 : "memory", "m0");
}
