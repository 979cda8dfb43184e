// Device-side building blocks shared by the attention kernels: vector types, MFMA
// wrappers for gfx950, the transposing LDS reads, and wavefront helpers.
//
// Register layouts used throughout (64-lane wavefront, lane l, col = l % 32, half = l / 32):
//   v_mfma_f32_32x32x16_{bf16,f16}: an A (or B) operand lane holds row (col) `l % 32` and the
//     8 contraction indices 8*half .. 8*half+7; the fp32 result lane holds column `l % 32`
//     and, in register r of 16, row 8*(r/4) + 4*half + r%4.
// Computing the transposed score tile S^T = K Q^T therefore leaves one query per lane
// column with its keys spread over the lane's own registers, and those registers, packed
// to 16 bits, are already a valid B operand for O^T = V^T P^T as long as the V operand
// enumerates keys in the same order -- the gfx950 counterpart of the accumulator-to-operand
// register permutation of the paper's section 3.3 (FP8 layout discussion).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>

namespace fa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

struct bf16_tag {};
struct f16_tag {};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <typename Tag> struct Elem;

template <> struct Elem<bf16_tag> {
    // D = A(32x16) * B(16x32) + C, 16-bit operands packed 8 per lane in a 128-bit carrier
    static __device__ __forceinline__ f32x16 mma(i32x4 a, i32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ int pack2(float lo, float hi) {  // RNE
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(int, __builtin_convertvector(v, bf16x2));
    }
    static __device__ __forceinline__ float to_float(uint16_t bits) {
        return __builtin_bit_cast(float, (uint32_t)bits << 16);
    }
};

template <> struct Elem<f16_tag> {
    static __device__ __forceinline__ f32x16 mma(i32x4 a, i32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ int pack2(float lo, float hi) {  // RNE
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(int, __builtin_convertvector(v, f16x2));
    }
    static __device__ __forceinline__ float to_float(uint16_t bits) {
        return (float)__builtin_bit_cast(_Float16, bits);
    }
};

// The same MFMA written as inline assembly, to choose the half of the register file each operand
// lives in.  A kernel that needs more than 256 registers per lane gets MFMA results in the
// accumulation half by default, where no VALU instruction can read them: a score tile that the
// softmax reads would pay one copy per element.  Here the accumulator is forced into ordinary
// registers and the B operand (touched by MFMA alone) is taken from the accumulation half.
// The compiler's hazard checker cannot see inside: a VALU read of the accumulator must be
// separated from the MFMA that wrote it by mfma_result_wait().
template <typename Tag> struct MfmaVgprAcc;
#define FA_DEFINE_MFMA_VGPR_ACC(TAG, OPCODE)                                                          \
    template <> struct MfmaVgprAcc<TAG> {                                                             \
        static __device__ __forceinline__ void run(f32x16& acc, const i32x4& a, const i32x4& b) {     \
            asm volatile(OPCODE " %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));                      \
        }                                                                                             \
        static __device__ __forceinline__ void first(f32x16& acc, const i32x4& a, const i32x4& b) {   \
            asm volatile(OPCODE " %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b));                      \
        }                                                                                             \
    };
FA_DEFINE_MFMA_VGPR_ACC(bf16_tag, "v_mfma_f32_32x32x16_bf16")
FA_DEFINE_MFMA_VGPR_ACC(f16_tag, "v_mfma_f32_32x32x16_f16")
#undef FA_DEFINE_MFMA_VGPR_ACC

// 13 wait states: the 8-pass MFMA needs 11 between its issue and a VALU read of its result, and
// the compiler leaves 12 or more in the code it schedules itself.  The accumulators are operands
// of the statement, so no reader can be scheduled above it; placed after an independent MFMA
// most of the wait passes while the matrix pipe works on that one.
static __device__ __forceinline__ void mfma_result_wait(f32x16& x, f32x16& y) {
    asm volatile("s_nop 12" : "+v"(x), "+v"(y));
}
static __device__ __forceinline__ void mfma_result_wait(f32x16& x) { asm volatile("s_nop 12" : "+v"(x)); }

// 32-bit LDS byte address of a __shared__ object, and loads through such an address: a base kept
// in one register with compile-time offsets lets every read use the instruction's immediate
// offset field instead of an address computation of its own.
static __device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)p; }
static __device__ __forceinline__ i32x4 lds_load_16B(uint32_t addr) {
    typedef i32x4 __attribute__((address_space(3))) * lds_vec_ptr;
    return *(lds_vec_ptr)(uintptr_t)addr;
}
static __device__ __forceinline__ f32x4 lds_load_4f(uint32_t addr) {
    typedef f32x4 __attribute__((address_space(3))) * lds_vec_ptr;
    return *(lds_vec_ptr)(uintptr_t)addr;
}

// ds_read_b64_tr_b16: the 16 lanes of a group each point at 4 consecutive 16-bit elements;
// seen as a 4x16 matrix (row r = what lanes 4r..4r+3 point at), lane i of the group
// receives column i.  Used to read a [key][d] tile as the key-contiguous MFMA operand.
static __device__ __forceinline__ i32x2 lds_read_tr16(const void* lds_ptr) {
    typedef s16x4 __attribute__((address_space(3))) * lds_vec_ptr;
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_vec_ptr)(uintptr_t)lds_ptr);
    return __builtin_bit_cast(i32x2, v);
}
static __device__ __forceinline__ i32x2 lds_read_tr16(uint32_t lds_addr) {
    typedef s16x4 __attribute__((address_space(3))) * lds_vec_ptr;
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_vec_ptr)(uintptr_t)lds_addr);
    return __builtin_bit_cast(i32x2, v);
}

// ds_read_b64_tr_b8: same with bytes; the group's data is an 8x16 byte matrix (row r = what
// lanes 2r, 2r+1 point at) and lane i receives column i.
static __device__ __forceinline__ i32x2 lds_read_tr8(const void* lds_ptr) {
    typedef i32x2 __attribute__((address_space(3))) * lds_vec_ptr;
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_vec_ptr)(uintptr_t)lds_ptr);
}
static __device__ __forceinline__ i32x2 lds_read_tr8(uint32_t lds_addr) {
    typedef i32x2 __attribute__((address_space(3))) * lds_vec_ptr;
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_vec_ptr)(uintptr_t)lds_addr);
}

// v_permlane32_swap exchanges the upper half of its first register with the lower half of
// its second.  Fed two copies of x it yields (x of lanes 0..31 replicated, x of lanes 32..63
// replicated).  The second copy is laundered through an empty asm so the compiler cannot
// treat the two results as one value.
struct HalfPair {
    float lo, hi;  // value of lane (l % 32), value of lane (l % 32) + 32
};
static __device__ __forceinline__ HalfPair both_halves(float x) {
    uint32_t a = __builtin_bit_cast(uint32_t, x);
    uint32_t b = a;
    asm volatile("" : "+v"(b));
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    uint32_t r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    return {__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}

static __device__ __forceinline__ float max_both_halves(float x) {
    HalfPair p = both_halves(x);
    return fmaxf(p.lo, p.hi);
}

static __device__ __forceinline__ float sum_both_halves(float x) {
    HalfPair p = both_halves(x);
    return p.lo + p.hi;
}

// Raw buffer access to a caller tensor: reads past `bytes` return zero instead of faulting.
static __device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buffer(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
static __device__ __forceinline__ i32x4 buffer_load_16B(__amdgpu_buffer_rsrc_t rsrc, int byte_off) {
    return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 0));
}

// Asynchronous global -> LDS copy of 16 bytes per lane (buffer load with an LDS destination):
// lane i's bytes land at lds_base + 16 i, lds_base wave-uniform; reads past the resource's size
// store zeros.  Written as inline assembly on purpose: the compiler then does not know that the
// load writes LDS and does not drain all outstanding loads before every later LDS read; the
// caller orders the two with an explicit vmcnt wait and a barrier.
struct BufferWords {
    i32x4 w;
};
static __device__ __forceinline__ BufferWords make_buffer_words(const void* base, uint32_t bytes) {
    const uint64_t a = reinterpret_cast<uint64_t>(base);
    BufferWords b;
    b.w = i32x4{(int)(uint32_t)a, (int)(uint32_t)((a >> 32) & 0xFFFF), (int)bytes, 0x00020000};
    return b;
}
static __device__ __forceinline__ void global_to_lds_16B(const BufferWords& rsrc, uint32_t lds_base, int byte_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(byte_off), "s"(rsrc.w)
                 : "memory", "m0");
}

static __device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Stores a wave's 32-row x (32 DT)-column fp32 accumulator tile (MFMA result layout with rows as
// lane columns: lane (col, half) holds row `col`; register r of tile dt is column
// 32 dt + 8 (r / 4) + 4 half + r % 4) as 16-bit elements, scaled by `factor`.  Stored straight from
// that layout every store instruction would touch 32 rows with 16 bytes each; instead the tile
// goes through `patch` (4 KiB of LDS private to the wave), 128 bytes of every row at a time, and
// leaves as whole 128-byte lines: 16-byte chunk c of row r sits at chunk c ^ (r % 8) of the patch.
// `rsrc` covers the [rows][32 DT] destination; rows at or past its end are dropped by the hardware.
template <typename Tag, int DT>
static __device__ __forceinline__ void store_rows_via_lds(const f32x16 (&acc)[DT], float factor, char* patch,
                                                           __amdgpu_buffer_rsrc_t rsrc, int row0, int lane) {
    static_assert(DT % 2 == 0, "128 bytes of a row are two 32-column tiles");
    using E = Elem<Tag>;
    constexpr int ROWB = DT * 64;  // bytes per destination row
    const int col = lane & 31, half = lane >> 5;
#pragma unroll
    for (int hd = 0; hd < DT / 2; ++hd) {
#pragma unroll
        for (int d2 = 0; d2 < 2; ++d2)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int dt = 2 * hd + d2;
                i32x2 w;
                w[0] = E::pack2(acc[dt][4 * g] * factor, acc[dt][4 * g + 1] * factor);
                w[1] = E::pack2(acc[dt][4 * g + 2] * factor, acc[dt][4 * g + 3] * factor);
                *reinterpret_cast<i32x2*>(patch + col * 128 + (((4 * d2 + g) ^ (col & 7)) << 4) + 8 * half) = w;
            }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 8 * i + (lane >> 3), pc = lane & 7;
            const i32x4 w = *reinterpret_cast<const i32x4*>(patch + r * 128 + (pc << 4));
            __builtin_amdgcn_raw_buffer_store_b128(w, rsrc, (row0 + r) * ROWB + hd * 128 + ((pc ^ (r & 7)) << 4), 0, 0);
        }
    }
}

// The chip deals consecutive workgroup ids round-robin to its 8 XCDs, each with a private
// L2.  Remap a linear id so that ids landing on one XCD cover a contiguous range of work
// items (all query tiles of a head share that head's K and V in one L2).
static __device__ __forceinline__ int xcd_contiguous(int id, int total) {
    constexpr int kXcd = 8;
    if (total % kXcd != 0) return id;
    return (id % kXcd) * (total / kXcd) + id / kXcd;
}

// Measurement builds (-DFA_CLOCK_SPAN): how many shader-clock cycles a launch took on one CU.  A kernel
// declares a ClockSpan as its first statement; workgroups that run on the chosen CU record the earliest
// entry stamp and the latest exit stamp (the shader clock is only comparable within a CU).  The CU is that
// of workgroup 0 of the first launch after the library is loaded, so that launch only chooses and the
// launches after it measure.  Cycles divided by the launch's wall time is the clock the chip actually ran
// at: it lowers the clock under load, so a kernel that needs fewer cycles need not take less time.  Each
// source file that holds measured kernels defines its reader with FA_CLOCK_SPAN_READER(name).  In ordinary
// builds ClockSpan is empty and generates no code.
#ifdef FA_CLOCK_SPAN
static __device__ unsigned long long fa_clock_span_cycles[2] = {~0ull, 0ull};
static __device__ int fa_clock_span_cu = -1;
struct ClockSpan {
    long long t0;
    __device__ __forceinline__ ClockSpan() : t0(__builtin_readcyclecounter()) {}
    __device__ __forceinline__ ~ClockSpan() {
        if (threadIdx.x == 0) {
            // XCC id, then shader engine / shader array / CU from the hardware id register
            const int cu = (int)(((__builtin_amdgcn_s_getreg((31 << 11) | 20) & 15) << 8) |
                                 ((__builtin_amdgcn_s_getreg((31 << 11) | 4) >> 8) & 255));
            if (blockIdx.x == 0 && fa_clock_span_cu < 0) fa_clock_span_cu = cu;
            if (cu == fa_clock_span_cu) {
                atomicMin(&fa_clock_span_cycles[0], (unsigned long long)t0);
                atomicMax(&fa_clock_span_cycles[1], (unsigned long long)__builtin_readcyclecounter());
            }
        }
    }
};
// span[0], span[1]: first entry and last exit stamp since the last call; the call clears them
#define FA_CLOCK_SPAN_READER(name)                                                                              \
    extern "C" int name(unsigned long long* span) {                                                             \
        const unsigned long long init[2] = {~0ull, 0ull};                                                       \
        if (hipDeviceSynchronize() != hipSuccess) return 1;                                                     \
        if (hipMemcpyFromSymbol(span, HIP_SYMBOL(fa::fa_clock_span_cycles), sizeof(init)) != hipSuccess) return 2; \
        return hipMemcpyToSymbol(HIP_SYMBOL(fa::fa_clock_span_cycles), init, sizeof(init)) == hipSuccess ? 0 : 3; \
    }
#else
struct ClockSpan {};
#define FA_CLOCK_SPAN_READER(name)
#endif

}  // namespace fa
