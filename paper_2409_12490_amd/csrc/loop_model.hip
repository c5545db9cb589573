// A diagnostic, not part of the attention path: model kernels of the bf16 attention key loop, used to
// separate what the instruction mix costs in cycles from what the chip's clock does under it.
//
//   kind 0   nothing but 32x32x16 bf16 MFMAs (32 per wave and step, 8 waves per compute unit)
//   kind 1   the key loop of attn_bf16.hip without its global traffic: per wave and step 16 K fragments
//            (ds_read_b128) + 16 V fragments (ds_read_b64_tr_b16 pairs) feeding 32 MFMAs, the softmax
//            arithmetic of a 32 x 64 tile (max, exp2, bf16 conversion, row sum by plain additions), waves
//            0-3 "matrix phase then softmax", waves 4-7 "softmax then matrix phase", one barrier per step
//   kind 2   kind 1 with the row sum through v_dot2c_f32_bf16 (which does not run beside the partner wave's
//            MFMAs)
//   random_bits 0 / 1   LDS contents and Q fragments are the constant 1.0 / pseudo-random bf16 values in
//            (-2, 2): the cycle counts are the same, the clock the chip sustains is not.
//
// Built into its own small library (libcp_loop_model.so); `python -m paper_2409_12490_amd.studies clock`
// runs it, under rocprofv3 --pmc GRBM_GUI_ACTIVE the counter divided by the duration gives the clock.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define RD128(d, addr, OFF) asm volatile("ds_read_b128 %0, %1 offset:" #OFF : "=v"(d) : "v"(addr))
#define RDTR(d, addr, OFF) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:" #OFF : "=v"(d) : "v"(addr))
#define WAIT4(n, a) asm volatile("s_waitcnt lgkmcnt(" #n ")" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]))
#define FENCE() __builtin_amdgcn_sched_barrier(0)

__device__ __forceinline__ unsigned mix(unsigned h) {
    h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
    return h;
}

template <int KIND, int RANDOM>
__global__ __launch_bounds__(512) void loop_model_kernel(float* sink, int steps) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) {
        const unsigned h = mix((i * 2654435761u) ^ (blockIdx.x * 40503u));
        // two bf16 per word: random sign and mantissa, exponent 0x7e or 0x7f
        ((unsigned*)smem)[i] = RANDOM ? ((h & 0x807f807fu) | 0x3f003f00u | ((h >> 3) & 0x00800080u)) : 0x3f803f80u;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, l32 = lane & 31, hh = lane >> 5;
    const unsigned lds0 = (unsigned)(size_t)smem;
    unsigned kaddr = lds0 + l32 * 256 + (((l32 & 15) ^ hh) << 4);
    const int i16 = lane & 15, gbit = (lane >> 4) & 1;
    unsigned vaddr = lds0 + 36864 + (4 * hh + (i16 >> 2)) * 256 +
                     ((((unsigned)(i16 >> 2) << 2) + 2 * gbit + ((i16 & 3) >> 1)) << 4) + (i16 & 1) * 8;
    bf16x8 qf;
    for (int j = 0; j < 8; ++j) {
        const unsigned h = mix((threadIdx.x * 8u + j) * 2246822519u);
        qf[j] = RANDOM ? (__bf16)(((int)(h & 255) - 128) * (1.0f / 128.0f)) : (__bf16)1.0f;
    }
    f32x16 s0 = {0}, s1 = {0}, o0 = {0}, o1 = {0}, o2 = {0}, o3 = {0};
    u32x4 ka[4], kb[4];                   // two groups of four K fragments
    u32x2 va[8], vb[8];                   // two groups of four V fragments (two halves each)
    // kind 0 never reads LDS: its A operands keep these register values
    auto word = [&](unsigned salt) {
        const unsigned h = mix((threadIdx.x * 64u + salt) * 2654435761u);
        return RANDOM ? ((h & 0x807f807fu) | 0x3f003f00u | ((h >> 3) & 0x00800080u)) : 0x3f803f80u;
    };
    for (int i = 0; i < 4; ++i) { ka[i] = (u32x4){word(4 * i), word(4 * i + 1), word(4 * i + 2), word(4 * i + 3)}; kb[i] = ka[i]; }
    for (int i = 0; i < 8; ++i) { va[i] = (u32x2){word(16 + 2 * i), word(17 + 2 * i)}; vb[i] = va[i]; }
    for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(ka[i]), "+v"(kb[i]));
    for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(va[i]), "+v"(vb[i]));
    constexpr bool LOOP = KIND != 0, DOT = KIND == 2;
    const bool rotated = (threadIdx.x >> 6) >= 4;          // shares its SIMD with wave - 4
    bf16x8 pf[4];
    for (int i = 0; i < 4; ++i) pf[i] = qf;
    float m_run = -1e30f, l_run = 0.f;

    auto softmax = [&]() {
        float mx = m_run;
        for (int r = 0; r < 16; r += 2) {
            mx = __builtin_fmaxf(__builtin_fmaxf(s0[r], s0[r + 1]), mx);
            mx = __builtin_fmaxf(__builtin_fmaxf(s1[r], s1[r + 1]), mx);
        }
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));
        if (__builtin_amdgcn_readfirstlane(__builtin_amdgcn_ballot_w64(mx > m_run + 8.f) != 0)) {
            const float al = __builtin_amdgcn_exp2f(m_run - mx);
            l_run *= al;
            for (int r = 0; r < 16; ++r) { o0[r] *= al; o1[r] *= al; o2[r] *= al; o3[r] *= al; }
            m_run = mx;
        }
        const float nm = -m_run * 0.125f;
        float rs = 0.f, rs2 = 0.f;
        bf16x2 one; one[0] = (__bf16)1.f; one[1] = (__bf16)1.f;
        for (int g = 0; g < 2; ++g) {
            f32x16& sv = g ? s1 : s0;
            for (int r = 0; r < 16; r += 2) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], 0.125f, nm));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r + 1], 0.125f, nm));
                bf16x2 pk; pk[0] = (__bf16)p0; pk[1] = (__bf16)p1;
                if (DOT) rs = __builtin_amdgcn_fdot2_f32_bf16(pk, one, rs, false);
                else { rs += p0; rs2 += p1; }
                pf[g * 2 + (r >> 3)][r & 7] = pk[0]; pf[g * 2 + (r >> 3)][(r & 7) + 1] = pk[1];
            }
        }
        l_run += rs + rs2;
    };
#define KGROUP(dst, ks) do { if (LOOP) { RD128(dst[0], kaddr, 0); RD128(dst[1], kaddr, 8192); RD128(dst[2], kaddr, 32); RD128(dst[3], kaddr, 8224); } kaddr ^= (ks); } while (0)
#define VGROUP(dst) do { if (LOOP) { RDTR(dst[0], vaddr, 0); RDTR(dst[1], vaddr, 2048); RDTR(dst[2], vaddr, 64); RDTR(dst[3], vaddr, 2112); RDTR(dst[4], vaddr, 128); RDTR(dst[5], vaddr, 2176); RDTR(dst[6], vaddr, 192); RDTR(dst[7], vaddr, 2240); } vaddr ^= 4096; } while (0)
#define KMFMA(src) do { s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, src[0]), qf, s0, 0, 0, 0); s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, src[1]), qf, s1, 0, 0, 0); \
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, src[2]), qf, s0, 0, 0, 0); s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, src[3]), qf, s1, 0, 0, 0); } while (0)
#define VF(src, i) __builtin_bit_cast(bf16x8, (u32x4){src[2 * (i)][0], src[2 * (i)][1], src[2 * (i) + 1][0], src[2 * (i) + 1][1]})
#define VMFMA(src, pi) do { o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(VF(src, 0), pf[pi], o0, 0, 0, 0); o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(VF(src, 1), pf[pi], o1, 0, 0, 0); \
      o2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(VF(src, 2), pf[pi], o2, 0, 0, 0); o3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(VF(src, 3), pf[pi], o3, 0, 0, 0); } while (0)
#define WAITK(n, x) do { if (LOOP) WAIT4(n, x); } while (0)
#define WAITV(n, x) do { if (LOOP) { WAIT4(n, x); asm volatile("" : "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])); } } while (0)
    KGROUP(ka, 64);
    for (int t = 0; t < steps; ++t) {
        if (LOOP && rotated) { softmax(); FENCE(); }
        if (LOOP) { for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; } }
        if (LOOP) __builtin_amdgcn_s_setprio(3);
        // K groups 0..3, then V groups 0..3; the next group's reads go out before the current group's MFMAs
        KGROUP(kb, 128); FENCE(); WAITK(4, ka); FENCE(); KMFMA(ka); FENCE();
        KGROUP(ka, 64); FENCE(); WAITK(4, kb); FENCE(); KMFMA(kb); FENCE();
        KGROUP(kb, 128 | 64); FENCE(); WAITK(4, ka); FENCE(); KMFMA(ka); FENCE();
        VGROUP(va); FENCE(); WAITK(8, kb); FENCE(); KMFMA(kb); FENCE();
        VGROUP(vb); FENCE(); WAITV(8, va); FENCE(); VMFMA(va, 0); FENCE();
        VGROUP(va); FENCE(); WAITV(8, vb); FENCE(); VMFMA(vb, 1); FENCE();
        VGROUP(vb); FENCE(); WAITV(8, va); FENCE(); VMFMA(va, 2); FENCE();
        KGROUP(ka, 64); FENCE(); WAITV(4, vb); FENCE(); VMFMA(vb, 3); FENCE();
        if (LOOP) __builtin_amdgcn_s_setprio(0);
        if (LOOP && !rotated) { softmax(); FENCE(); }
        if (LOOP) __syncthreads();
    }
    asm volatile("s_waitcnt lgkmcnt(0)");
    float acc = l_run + m_run;
    for (int r = 0; r < 16; ++r) acc += s0[r] + s1[r] + o0[r] + o1[r] + o2[r] + o3[r];
    if (acc == 12345.f) sink[0] = acc;                     // keeps the arithmetic alive; practically never true
}

static __device__ float loop_model_sink[4];

template <int KIND, int RANDOM>
hipError_t run_one(int steps, float* ms) {
    float* sink = nullptr;
    hipError_t e = hipGetSymbolAddress((void**)&sink, HIP_SYMBOL(loop_model_sink));
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)loop_model_kernel<KIND, RANDOM>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    hipEvent_t e0, e1;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return e;
    if ((e = hipEventCreate(&e1)) != hipSuccess) return e;
    hipLaunchKernelGGL((loop_model_kernel<KIND, RANDOM>), dim3(cus), dim3(512), 65536, 0, sink, 16);   // warm-up
    e = hipEventRecord(e0, 0);
    hipLaunchKernelGGL((loop_model_kernel<KIND, RANDOM>), dim3(cus), dim3(512), 65536, 0, sink, steps);
    if (e == hipSuccess) e = hipEventRecord(e1, 0);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    const hipError_t d0 = hipEventDestroy(e0), d1 = hipEventDestroy(e1);
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = d0 != hipSuccess ? d0 : d1;
    return e;
}

}  // namespace

// kind 0..2, random_bits 0/1 (see the head of this file); steps: 64-key steps per compute unit (one workgroup of 8
// waves per compute unit).  Writes the duration of the timed launch in milliseconds.  Returns 0, -1 for a bad argument,
// or a positive hipError_t.  Runs on the current device's default stream and synchronises.
extern "C" int cp_loop_model(int kind, int random_bits, int steps, float* milliseconds) {
    if (kind < 0 || kind > 2 || steps <= 0 || steps > (1 << 22) || !milliseconds) return -1;
    hipError_t e;
    const int r = random_bits ? 1 : 0;
    if (kind == 0) e = r ? run_one<0, 1>(steps, milliseconds) : run_one<0, 0>(steps, milliseconds);
    else if (kind == 1) e = r ? run_one<1, 1>(steps, milliseconds) : run_one<1, 0>(steps, milliseconds);
    else e = r ? run_one<2, 1>(steps, milliseconds) : run_one<2, 0>(steps, milliseconds);
    return (int)e;
}
