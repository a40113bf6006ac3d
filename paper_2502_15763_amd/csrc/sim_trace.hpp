// Canonical run-length trace of the iteration simulators and its FNV-1a hash (gfx950, wave64):
// records (kind u32, count u32, t_start i64, x i64); consecutive decode iterations with equal D
// merge into one record.  Shared by the FCFS simulator and the assigned-queue simulator.
#pragma once
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr uint64_t kFnvBasis = 0xcbf29ce484222325ull;
constexpr uint64_t kFnvPrime = 0x100000001b3ull;

__device__ __forceinline__ int64_t uniform_i64(int64_t x)
{
    uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)x >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Wave sum and inclusive wave scan of token counts 0 <= x < 2^33 (up to four input lengths per lane):
// the low 24 bits and the bits above them go through 32-bit DPP reductions, which replaces twelve
// dependent LDS permutes of a 64-bit shuffle reduction by twelve DPP adds.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t x)
{
    uint32_t v = x;
    v += dpp_u32<0x111, 0xf>(0u, v);           // row_shr 1, 2, 4, 8: inclusive prefix inside each row of 16
    v += dpp_u32<0x112, 0xf>(0u, v);
    v += dpp_u32<0x114, 0xf>(0u, v);
    v += dpp_u32<0x118, 0xf>(0u, v);
    v += dpp_u32<0x142, 0xa>(0u, v);           // row_bcast:15: rows 1 and 3 add the total of the row before
    v += dpp_u32<0x143, 0xc>(0u, v);           // row_bcast:31: rows 2 and 3 add the total of rows 0 and 1
    return v;
}

__device__ __forceinline__ int64_t wave_sum_tokens(int64_t x)
{
    const uint32_t lo = (uint32_t)x & 0xFFFFFFu, hi = (uint32_t)((uint64_t)x >> 24);
    return (int64_t)(((uint64_t)wave_sum_u32(hi) << 24) + (uint64_t)wave_sum_u32(lo));
}

__device__ __forceinline__ int64_t wave_incl_scan_tokens(int64_t x)
{
    const uint32_t lo = (uint32_t)x & 0xFFFFFFu, hi = (uint32_t)((uint64_t)x >> 24);
    return (int64_t)(((uint64_t)wave_incl_scan_u32(hi) << 24) + (uint64_t)wave_incl_scan_u32(lo));
}

// 64-bit division is a long instruction sequence: one copy, out of line, keeps the simulator loops compact
// (they run from the instruction cache with eight waves per SIMD at different places).
__device__ __attribute__((noinline)) uint64_t udiv64(uint64_t a, uint64_t b) { return a / b; }

// Products of wave-uniform operands on the scalar unit, written out in 32-bit pieces: a 64 x 64-bit
// product whose operands are known to be narrow still costs the full expansion (the zero halves are
// multiplied too), and scalar issue is what bounds the simulators.
__device__ __forceinline__ uint32_t s_mul_hi(uint32_t a, uint32_t b)
{
    // (the operands are wave-uniform; readfirstlane pins them to scalar registers even where the compiler
    //  cannot prove that, and costs nothing where it can)
    const uint32_t sa = (uint32_t)__builtin_amdgcn_readfirstlane((int)a), sb = (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
    uint32_t r;
    asm("s_mul_hi_u32 %0, %1, %2" : "=s"(r) : "s"(sa), "s"(sb));
    return r;
}
// a * b for 32-bit a and b: two instructions
__device__ __forceinline__ int64_t mul_u32_u32(uint32_t a, uint32_t b)
{
    return (int64_t)(((uint64_t)s_mul_hi(a, b) << 32) | (uint64_t)(a * b));
}
// a * b modulo 2^64 for a 32-bit a: four instructions
__device__ __forceinline__ int64_t mul_u32_i64(uint32_t a, int64_t b)
{
    const uint32_t bl = (uint32_t)(uint64_t)b, bh = (uint32_t)((uint64_t)b >> 32);
    const uint32_t hi = s_mul_hi(a, bl) + a * bh;
    return (int64_t)(((uint64_t)hi << 32) | (uint64_t)(a * bl));
}

template <int NBYTES>
__device__ __forceinline__ uint64_t fnv_plain(uint64_t h, uint64_t w)
{
#pragma unroll
    for (int b = 0; b < NBYTES; b++) {
        h = (h ^ (w & 0xffull)) * kFnvPrime;
        w >>= 8;
    }
    return h;
}

// the byte-by-byte form of the record hash: rare, kept out of line so that the loops stay compact
__device__ __attribute__((noinline)) uint64_t fnv_record_wide(uint64_t h, uint32_t kind, uint32_t count, uint64_t ut, uint64_t ux)
{
    h = fnv_plain<8>(h, (uint64_t)kind | ((uint64_t)count << 32));
    h = fnv_plain<8>(h, ut);
    return fnv_plain<8>(h, ux);
}

// FNV-1a of one 24-byte trace record (kind u32, count u32, t_start i64, x i64, little endian).
//
// A byte step is (hi:lo) <- ((hi:lo) ^ b) * prime.  The xor only touches lo, and the z zero bytes
// that follow a byte only multiply by prime^z more, so a byte together with the zeros after it is one step
//     v = lo ^ b;   lo' = v * Pl;   hi' = hi * Pl + v * Ph + mulhi(v, Pl)      (Ph:Pl = prime^(1+z))
// The lo chain is the only sequential part (xor, multiply).  hi is linear in the v of the steps:
// hi_end = hi_0 * prod(Pl) + sum_s e_s * W_s,  e_s = v_s * Ph_s + mulhi(v_s, Pl_s), W_s = product of the
// Pl of the later steps.  Every lane runs the lo chain on the vector unit (measured: with the chain on the
// scalar unit, whole or one record of two, the simulators are 4 to 7 % slower, the scalar unit being the
// busier one in their loops); the four lanes of group s keep v_s (one DPP move under a row and bank mask
// per step), one lane of the group holds the step's constants, and one wave sum finishes the record.
// Trace fields are small numbers in wide words; for count < 2^16, 0 <= t_start < 2^40 and
// 0 <= x < 2^16 the record is the fixed sequence of 10 steps below (bytes known to be zero are
// folded into the step of the byte before them).  Anything else takes the byte-by-byte path.
constexpr uint64_t fnv_pow(int z) { uint64_t r = 1; for (int i = 0; i < z; i++) r *= kFnvPrime; return r; }
constexpr int kHashSteps = 10;
constexpr int kStepBytes[kHashSteps] = {4, 1, 3, 1, 1, 1, 1, 4, 1, 7};   // kind + 0*3, count, count + 0*2, t*4, t + 0*3, x, x + 0*6
constexpr int step_after(int s) { int n = 24; for (int i = 0; i <= s; i++) n -= kStepBytes[i]; return n; }

struct HashLane {          // per-lane constants of the record hash (lane 16 (s / 4) + 4 (s % 4) + 3 = step s; zero elsewhere)
    uint32_t pl, ph, w, w24;   // w24 = w * prime^24: the weight of a step when one more record follows in the same sum
};

__device__ __forceinline__ HashLane hash_lane_init(int lane)
{
    HashLane c;
    c.pl = 0; c.ph = 0; c.w = 0; c.w24 = 0;
#pragma unroll
    for (int st = 0; st < kHashSteps; st++)
        if (lane == 16 * (st / 4) + 4 * (st % 4) + 3) {
            c.pl = (uint32_t)fnv_pow(kStepBytes[st]);
            c.ph = (uint32_t)(fnv_pow(kStepBytes[st]) >> 32);
            c.w = (uint32_t)fnv_pow(step_after(st));
            c.w24 = (uint32_t)fnv_pow(step_after(st) + 24);
        }
    return c;
}

// Keeps v in the four lanes of group G (row G / 4, bank G % 4) of x: one DPP move under a row and bank mask.
template <int G>
__device__ __forceinline__ uint32_t keep_in_group(uint32_t x, uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)v, 0xE4, 1 << (G / 4), 1 << (G % 4), false);
}

__device__ __forceinline__ uint64_t fnv_record(uint64_t h, uint32_t kind, uint32_t count, int64_t t_start, int64_t x,
                                               const HashLane &c)
{
    const uint64_t ut = (uint64_t)t_start, ux = (uint64_t)x;
    if (__builtin_expect(((uint64_t)(count >> 16) | (ut >> 40) | (ux >> 16) | (uint64_t)(kind >> 8)) != 0, 0))
        return fnv_record_wide(h, kind, count, ut, ux);
    uint32_t lo = (uint32_t)h, hi = (uint32_t)(h >> 32);
    asm("" : "+v"(lo));            // the chain stays in vector registers
    uint32_t vv = 0;
    constexpr uint32_t kP1 = (uint32_t)fnv_pow(1), kP3 = (uint32_t)fnv_pow(3), kP4 = (uint32_t)fnv_pow(4),
                       kP7 = (uint32_t)fnv_pow(7), kP24 = (uint32_t)fnv_pow(24);
    const uint32_t tl = (uint32_t)ut, th = (uint32_t)(ut >> 32);
#define MMBP_STEP(ST, B, PL) do { const uint32_t v_ = lo ^ (B); vv = keep_in_group<ST>(vv, v_); lo = v_ * (PL); } while (0)
    MMBP_STEP(0, kind, kP4);
    MMBP_STEP(1, count & 0xffu, kP1);
    MMBP_STEP(2, count >> 8, kP3);
    MMBP_STEP(3, tl & 0xffu, kP1);
    MMBP_STEP(4, (tl >> 8) & 0xffu, kP1);
    MMBP_STEP(5, (tl >> 16) & 0xffu, kP1);
    MMBP_STEP(6, tl >> 24, kP1);
    MMBP_STEP(7, th, kP4);
    MMBP_STEP(8, (uint32_t)ux & 0xffu, kP1);
    MMBP_STEP(9, (uint32_t)ux >> 8, kP7);
#undef MMBP_STEP
    uint32_t e = (vv * c.ph + __umulhi(vv, c.pl)) * c.w;
    e += dpp_u32<0x114, 0xf>(0u, e);           // lanes 3, 7, 11, 15 of a row hold its terms: row_shr 4 and 8 sum them
    e += dpp_u32<0x118, 0xf>(0u, e);           // into lane 15, the two row broadcasts carry the rows into lane 63
    e += dpp_u32<0x142, 0xa>(0u, e);
    e += dpp_u32<0x143, 0xc>(0u, e);
    hi = hi * kP24 + (uint32_t)__builtin_amdgcn_readlane((int)e, 63);
    return ((uint64_t)hi << 32) | lo;
}

// Two records in a row (a decode run and the prefill after it, the usual pair): the lo chain runs through both,
// and their hi terms meet in one wave sum.
__device__ __forceinline__ uint64_t fnv_record_pair(uint64_t h, uint32_t kind1, uint32_t count1, int64_t t1, int64_t x1,
                                                    uint32_t kind2, uint32_t count2, int64_t t2, int64_t x2, const HashLane &c)
{
    const uint64_t ut1 = (uint64_t)t1, ux1 = (uint64_t)x1, ut2 = (uint64_t)t2, ux2 = (uint64_t)x2;
    if (__builtin_expect(((uint64_t)(count1 >> 16) | (ut1 >> 40) | (ux1 >> 16) | (uint64_t)(kind1 >> 8) |
                          (uint64_t)(count2 >> 16) | (ut2 >> 40) | (ux2 >> 16) | (uint64_t)(kind2 >> 8)) != 0, 0))
        return fnv_record(fnv_record(h, kind1, count1, t1, x1, c), kind2, count2, t2, x2, c);
    uint32_t lo = (uint32_t)h, hi = (uint32_t)(h >> 32);
    asm("" : "+v"(lo));
    uint32_t va = 0, vb = 0;
    constexpr uint32_t kP1 = (uint32_t)fnv_pow(1), kP3 = (uint32_t)fnv_pow(3), kP4 = (uint32_t)fnv_pow(4),
                       kP7 = (uint32_t)fnv_pow(7), kP48 = (uint32_t)fnv_pow(48);
#define MMBP_STEP(VV, ST, B, PL) do { const uint32_t v_ = lo ^ (B); VV = keep_in_group<ST>(VV, v_); lo = v_ * (PL); } while (0)
#define MMBP_RECORD(VV, KIND, COUNT, UT, UX) do { \
        const uint32_t tl_ = (uint32_t)(UT), th_ = (uint32_t)((UT) >> 32); \
        MMBP_STEP(VV, 0, KIND, kP4); \
        MMBP_STEP(VV, 1, (COUNT) & 0xffu, kP1); \
        MMBP_STEP(VV, 2, (COUNT) >> 8, kP3); \
        MMBP_STEP(VV, 3, tl_ & 0xffu, kP1); \
        MMBP_STEP(VV, 4, (tl_ >> 8) & 0xffu, kP1); \
        MMBP_STEP(VV, 5, (tl_ >> 16) & 0xffu, kP1); \
        MMBP_STEP(VV, 6, tl_ >> 24, kP1); \
        MMBP_STEP(VV, 7, th_, kP4); \
        MMBP_STEP(VV, 8, (uint32_t)(UX) & 0xffu, kP1); \
        MMBP_STEP(VV, 9, (uint32_t)(UX) >> 8, kP7); \
    } while (0)
    MMBP_RECORD(va, kind1, count1, ut1, ux1);
    MMBP_RECORD(vb, kind2, count2, ut2, ux2);
#undef MMBP_RECORD
#undef MMBP_STEP
    uint32_t e = (va * c.ph + __umulhi(va, c.pl)) * c.w24 + (vb * c.ph + __umulhi(vb, c.pl)) * c.w;
    e += dpp_u32<0x114, 0xf>(0u, e);
    e += dpp_u32<0x118, 0xf>(0u, e);
    e += dpp_u32<0x142, 0xa>(0u, e);
    e += dpp_u32<0x143, 0xc>(0u, e);
    hi = hi * kP48 + (uint32_t)__builtin_amdgcn_readlane((int)e, 63);
    return ((uint64_t)hi << 32) | lo;
}

// TRACED = false: the caller asked for no trace records, so none of the code that would store them exists.
template <bool TRACED = true>
struct Trace {
    uint64_t h;
    HashLane hc;
    mmbp_trace_rec *buf;
    int cap, len;
    int run_open;
    uint32_t run_count;
    int64_t run_t, run_D;

    __device__ __forceinline__ void emit(uint32_t kind, uint32_t count, int64_t t_start, int64_t x, int lane)
    {
        h = fnv_record(h, kind, count, t_start, x, hc);
        if constexpr (TRACED) {
            if (buf && len < cap && lane == 0) {
                mmbp_trace_rec r;
                r.kind = kind; r.count = count; r.t_start = t_start; r.x = x;
                buf[len] = r;
            }
        }
        // (counted in a vector register: nothing in the untraced loop reads it back, so it takes no scalar slot)
        { int one = 1; asm("" : "+v"(one)); len += one; }
    }
    __device__ __forceinline__ void flush(int lane)
    {
        if (run_open) { emit(0u, run_count, run_t, run_D, lane); run_open = 0; }
    }
    // k consecutive decode iterations with D running requests, the first starting at t
    __device__ __forceinline__ void decode(int64_t t, int64_t D, uint32_t k, int lane)
    {
        if (run_open && run_D == D) { run_count += k; return; }
        flush(lane);
        run_open = 1; run_count = k; run_t = t; run_D = D;
    }
    __device__ __forceinline__ void other(uint32_t kind, uint32_t count, int64_t t, int64_t x, int lane)
    {
        if constexpr (!TRACED) {
            if (run_open) {                      // the open decode run and this record in one go
                h = fnv_record_pair(h, 0u, run_count, run_t, run_D, kind, count, t, x, hc);
                run_open = 0;
                { int two = 2; asm("" : "+v"(two)); len += two; }
                return;
            }
        }
        flush(lane);
        emit(kind, count, t, x, lane);
    }
};

}  // namespace
}  // namespace mmbp
