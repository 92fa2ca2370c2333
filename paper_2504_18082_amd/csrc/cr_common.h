// Shared host/device helpers of libcommrand.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/commrand.h"

// host-side handle behind the C ABI's cr_ctx
struct cr_ctx {
    int32_t device;
    uint32_t flags;
    int64_t *status;        // device int64[CR_CTX_STATUS_WORDS], caller-owned, or NULL
};

namespace cr {

// ---- host side: error text, dry-run flag, argument checks ------------------------------------
void set_error(const char *fmt, ...);
bool dry_run();             // the calling thread's current context asks for validation only
int64_t *async_status();    // device status words of the calling thread's current context, or NULL

#define CR_REQUIRE(cond, code, ...)                  \
    do {                                             \
        if (!(cond)) {                               \
            ::cr::set_error(__VA_ARGS__);            \
            return (code);                           \
        }                                            \
    } while (0)

#define CR_HIP_CHECK(expr)                                                              \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) {                                                         \
            ::cr::set_error("%s failed: %s", #expr, hipGetErrorString(e_));             \
            return CR_ERR_HIP;                                                          \
        }                                                                               \
    } while (0)

#define CR_LAUNCH_CHECK()                                                               \
    do {                                                                                \
        hipError_t e_ = hipGetLastError();                                              \
        if (e_ != hipSuccess) {                                                         \
            ::cr::set_error("kernel launch failed: %s", hipGetErrorString(e_));         \
            return CR_ERR_HIP;                                                          \
        }                                                                               \
    } while (0)

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline int64_t ceil_div(int64_t x, int64_t m) { return (x + m - 1) / m; }

// carve an aligned slice out of a workspace
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T>
    T *take(size_t n)
    {
        off = (off + 255) & ~size_t(255);
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += n * sizeof(T);
        return p;
    }
    size_t bytes() const { return (off + 255) & ~size_t(255); }
};

// ---- device side ------------------------------------------------------------------------------
constexpr int WAVE = 64;

// Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> four words.
struct u32x4 { uint32_t x, y, z, w; };

// Both halves of a 32 x 32 bit product from ONE instruction (v_mad_u64_u32): the compiler splits a widening multiply
// into a high and a low multiply, which costs a fifth more per Philox block on this chip.
__device__ __forceinline__ void mul_hi_lo(uint32_t m, uint32_t c, uint32_t &hi, uint32_t &lo)
{
    uint64_t p;
    asm("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(p) : "v"(m), "v"(c) : "vcc");
    hi = (uint32_t)(p >> 32);
    lo = (uint32_t)p;
}

// a ^ b ^ c in one instruction (gfx950's three-input bit operation; truth table 0x96 is the parity of the three bits)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96); }

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        uint32_t hi0, lo0, hi1, lo1;
        mul_hi_lo(0xD2511F53u, c0, hi0, lo0);
        mul_hi_lo(0xCD9E8D57u, c2, hi1, lo1);
        // (first round: counter and key words are often the same for the whole wave, and their xor is then scalar work)
        c0 = i == 0 ? hi1 ^ (c1 ^ k0) : xor3(hi1, c1, k0);
        c1 = lo1;
        c2 = i == 0 ? hi0 ^ (c3 ^ k1) : xor3(hi0, c3, k1);
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return {c0, c1, c2, c3};
}

// stream domains (bits 4..7 of counter word 3)
constexpr uint32_t DOMAIN_COMMUNITY = 0, DOMAIN_NODE = 1, DOMAIN_NEIGHBOUR = 2;

__device__ __forceinline__ uint64_t shuffle_key(uint64_t seed, uint32_t epoch, uint32_t domain, uint32_t id)
{
    const u32x4 w = philox4x32_10(0u, id, 0u, (epoch << 8) | (domain << 4), (uint32_t)seed, (uint32_t)(seed >> 32));
    return ((uint64_t)w.x << 32) | w.y;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }

// float -> bf16 on raw bit patterns, round to nearest even, two values per instruction (gfx950 converts in hardware:
// v_cvt_pk_bf16_f32; infinities stay, NaNs stay NaNs)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2_t));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)(pack_bf16x2(f, 0.f) & 0xFFFFu); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// Block ids are dealt round-robin to the 8 XCDs, each with its own L2.  Give every XCD one
// contiguous range of logical tiles so that neighbouring tiles share a cache.
__device__ __forceinline__ uint32_t xcd_remap(uint32_t bid, uint32_t nblocks)
{
    constexpr uint32_t XCDS = 8;
    const uint32_t per = nblocks / XCDS;       // full rounds
    const uint32_t body = per * XCDS;
    if (bid >= body) return bid;               // ragged tail keeps its place
    return (bid % XCDS) * per + bid / XCDS;
}

// Same idea for grids sized by a capacity of which only the first `nwork` logical tiles exist (the
// count is read from a device-side header): the first 8 * ceil(nwork / 8) blocks share the tiles so that
// every XCD walks one contiguous range; returns false for a block that has no tile.
__device__ __forceinline__ bool xcd_compact(uint32_t bid, uint32_t nwork, uint32_t &logical)
{
    constexpr uint32_t XCDS = 8;
    const uint32_t per = (nwork + XCDS - 1) / XCDS;
    if (bid >= per * XCDS) return false;
    logical = (bid % XCDS) * per + bid / XCDS;
    return logical < nwork;
}

// ---------------------------------------------------------------------------------------------
// exclusive scan of one int per thread over a workgroup of NW waves (NW <= 16)
// ---------------------------------------------------------------------------------------------
template <int NW>
__device__ __forceinline__ int block_exclusive_scan(int x, int *lds /*[17]*/, int &total)
{
    const int lane = lane_id(), wave = threadIdx.x / WAVE;
    int incl = x;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
        const int y = __shfl_up(incl, off);
        if (lane >= off) incl += y;
    }
    if (lane == WAVE - 1) lds[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const int t = lane < NW ? lds[lane] : 0;
        int inc = t;
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            const int y = __shfl_up(inc, off);
            if (lane >= off) inc += y;
        }
        if (lane < NW) lds[lane] = inc - t;
        if (lane == 15) lds[16] = inc;
    }
    __syncthreads();
    total = lds[16];
    return lds[wave] + incl - x;
}

__device__ __forceinline__ int block_exclusive_scan_1024(int x, int *lds /*[17]*/, int &total)
{
    return block_exclusive_scan<16>(x, lds, total);
}

// out[0..n] = exclusive prefix sums of in[0..n) (out[n] = total), by one workgroup of 1024 threads.
// The input is walked in super-tiles of 1024 x 16 elements; a thread owns 16 consecutive elements of
// a super-tile and issues all of its loads before the first add.
__device__ __forceinline__ int scan_chunked(const int32_t *in, int32_t *out, int32_t *out_copy, int n, int *lds)
{
    constexpr int ITEMS = 16;
    int carry = 0;
    for (int tile0 = 0; tile0 < n; tile0 += 1024 * ITEMS) {
        const int start = tile0 + threadIdx.x * ITEMS;
        int x[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) x[i] = start + i < n ? in[start + i] : 0;
        int sum = 0;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) sum += x[i];
        int total;
        int run = carry + block_exclusive_scan_1024(sum, lds, total);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            if (start + i < n) {
                out[start + i] = run;
                if (out_copy) out_copy[start + i] = run;
            }
            run += x[i];
        }
        carry += total;
        __syncthreads();      // lds is reused by the next super-tile
    }
    if (threadIdx.x == 0) out[n] = carry;
    return carry;
}

}  // namespace cr
