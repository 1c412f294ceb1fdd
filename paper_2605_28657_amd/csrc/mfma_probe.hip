// Measurement aid, not part of the decode: what bf16 MFMA rate does this GPU sustain, and at which stage of
// operand delivery is it lost?  The convolution kernels of the decode are judged against the rate printed here
// as well as against the published peak, because under the board's power cap the published peak is not
// reachable with operands that toggle like real activations.
//
//   mfma_probe <mode> <seconds> <random>
//     mode 0: MFMAs on operands held in registers
//     mode 1: operands re-read from LDS for every MFMA group (the fragment reads of a 64 x 64 wave tile)
//     mode 2: the whole stage loop of a 128 x 128 x 64 tile: weight block global -> registers -> LDS, one
//             barrier per stage, fragment reads, MFMAs
//     mode 3: as mode 0 with the 16 x 16 x 32 MFMA shape (same FLOP count per wave)
//     mode 4: as mode 2 with the 16 x 16 x 32 MFMA shape (a 64 x 64 wave tile as 4 x 4 tiles)
//     mode 5: as mode 2 with one weight buffer in LDS and two barriers per stage (46 KB: three workgroups per CU)
//     mode 6: weight fragments straight from global memory into registers (fragment-major weights, two register sets),
//             activation fragments from LDS; no barrier in the stage loop
//     random 0: constant operands (little switching activity); 1: pseudo-random bf16 values of magnitude ~1
//
// Prints the rate of the first launch and the rate sustained over <seconds> of back-to-back launches; read the
// socket power and the shader clock beside it (hwmon power1_input, amd-smi metric -c).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

constexpr int MT = 128, NT = 128, WM = 2, WN = 2, NTH = 64 * WM * WN, KC = 64, LDK = KC + 8, SEGS = KC / 8;
constexpr int WTM = MT / WM, WTN = NT / WN, TM = WTM / 32, TN = WTN / 32;
constexpr int A_CH = MT * SEGS, A_ITERS = A_CH / NTH, XR = NT + 64;
constexpr int STAGES_PER_TILE = 56, N_TILES = 8;

__device__ __forceinline__ uint16_t hash_bf16(unsigned x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    // sign and 7 mantissa bits random, exponent 126 or 127: |value| in [0.5, 2)
    return (uint16_t)((x & 0x807fu) | (0x3f00u + ((x >> 20) & 0x0080u)));
}

template <int MODE, int RANDOM, bool S16 = false, int NB = 2>
__global__ __launch_bounds__(NTH) void probe_kernel(const uint16_t* w, float* out, int nstages, unsigned wbytes)
{
    __shared__ __attribute__((aligned(16))) uint16_t As[NB][MT * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Xs[XR * LDK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave / WN, wn = wave % WN, j = lane & 31, h = lane >> 5;
    for (int i = tid; i < NB * MT * LDK; i += NTH)
        (&As[0][0])[i] = RANDOM ? hash_bf16(i * 2654435761u + blockIdx.x) : (uint16_t)0x3c00;
    for (int i = tid; i < XR * LDK; i += NTH)
        Xs[i] = RANDOM ? hash_bf16(i * 40503u + 7u * blockIdx.x + 12345u) : (uint16_t)0x3c00;
    __syncthreads();
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(w), 0, (int)wbytes, 0x00020000);
    f32x16 acc[TM][TN];
    for (int a = 0; a < TM; ++a) for (int b = 0; b < TN; ++b) for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    u32x4 ra[A_ITERS];
    const unsigned tile0 = (blockIdx.x % N_TILES) * STAGES_PER_TILE * (A_CH * 16u);
    bf16x8 af[TM], bfr[TN];
    for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const bf16x8*>(&As[0][(wm * WTM + j + mi * 32) * LDK + h * 8]);
    for (int ni = 0; ni < TN; ++ni) bfr[ni] = *reinterpret_cast<const bf16x8*>(&Xs[(wn * WTN + j + ni * 32) * LDK + h * 8]);
    for (int stage = 0; stage < nstages; ++stage) {
        if (MODE == 2) {
            const unsigned base = tile0 + (unsigned)((stage + 1) % STAGES_PER_TILE) * (A_CH * 16u);
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it) ra[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, tid * 16u, base + it * (NTH * 16u), 0);
        }
        const int off = (stage % 7) * 9;                     // tap offsets of a dilation-9 convolution
        const uint16_t* abase = &As[stage & (NB - 1)][(wm * WTM + j) * LDK + h * 8];
        const int xoff = (wn * WTN + j + off) * LDK + h * 8;
        if constexpr (S16) {
            const int l16 = lane & 15, g4 = lane >> 4;
            f32x4* acc4 = reinterpret_cast<f32x4*>(&acc[0][0]);        // 16 tiles of 16 x 16
#pragma unroll
            for (int ks = 0; ks < KC / 32; ++ks) {
                bf16x8 a4[4], b4[4];
#pragma unroll
                for (int mi = 0; mi < 4; ++mi) a4[mi] = *reinterpret_cast<const bf16x8*>(&As[stage & (NB - 1)][(wm * WTM + mi * 16 + l16) * LDK + ks * 32 + g4 * 8]);
#pragma unroll
                for (int ni = 0; ni < 4; ++ni) b4[ni] = *reinterpret_cast<const bf16x8*>(&Xs[(wn * WTN + ni * 16 + l16 + off) * LDK + ks * 32 + g4 * 8]);
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 4; ++ni)
                        acc4[mi * 4 + ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a4[mi], b4[ni], acc4[mi * 4 + ni], 0, 0, 0);
            }
        } else
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            if (MODE >= 1) {
#pragma unroll
                for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const bf16x8*>(abase + mi * 32 * LDK + ks * 16);
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) bfr[ni] = *reinterpret_cast<const bf16x8*>(&Xs[xoff + ni * 32 * LDK + ks * 16]);
            }
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
        }
        if (MODE == 2) {
            if (NB == 1) __syncthreads();                     // every wave is done with the single weight buffer
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it) {
                const int q = tid + it * NTH;
                *reinterpret_cast<u32x4*>(&As[(stage + 1) & (NB - 1)][(q / SEGS) * LDK + (q % SEGS) * 8]) = ra[it];
            }
            __syncthreads();
        }
    }
    float s = 0;
    for (int a = 0; a < TM; ++a) for (int b = 0; b < TN; ++b) for (int r = 0; r < 16; ++r) s += acc[a][b][r];
    out[blockIdx.x * NTH + tid] = s;
}

// mode 6
template <int RANDOM>
__global__ __launch_bounds__(NTH) void probe_direct_kernel(const uint16_t* w, float* out, int nstages, unsigned wbytes)
{
    __shared__ __attribute__((aligned(16))) uint16_t Xs[XR * LDK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave / WN, wn = wave % WN, j = lane & 31, h = lane >> 5;
    for (int i = tid; i < XR * LDK; i += NTH)
        Xs[i] = RANDOM ? hash_bf16(i * 40503u + 7u * blockIdx.x + 12345u) : (uint16_t)0x3c00;
    __syncthreads();
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(w), 0, (int)wbytes, 0x00020000);
    f32x16 acc[TM][TN];
    for (int a = 0; a < TM; ++a) for (int b = 0; b < TN; ++b) for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    const unsigned tile0 = (blockIdx.x % N_TILES) * STAGES_PER_TILE * (A_CH * 16u);
    // a stage's 16 KB block holds 16 fragments of 1 KB: (wm, mi, ks); lane l reads its 16 bytes of each
    const unsigned voff = (unsigned)(wm * TM * (KC / 16)) * 1024u + lane * 16u;
    u32x4 fa[KC / 16][TM], fb[KC / 16][TM];
    auto load_frags = [&](u32x4 (&f)[KC / 16][TM], int stage) __attribute__((always_inline)) {
        const unsigned base = tile0 + (unsigned)(stage % STAGES_PER_TILE) * (A_CH * 16u);
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks)
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
                f[ks][mi] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, voff, base + (unsigned)(mi * (KC / 16) + ks) * 1024u, 0);
    };
    auto compute = [&](const u32x4 (&f)[KC / 16][TM], int stage) __attribute__((always_inline)) {
        const int off = (stage % 7) * 9;
        const int xoff = (wn * WTN + j + off) * LDK + h * 8;
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            bf16x8 bfr[TN];
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) bfr[ni] = *reinterpret_cast<const bf16x8*>(&Xs[xoff + ni * 32 * LDK + ks * 16]);
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f[ks][mi]), bfr[ni], acc[mi][ni], 0, 0, 0);
        }
    };
    load_frags(fa, 0);
    for (int stage = 0; stage < nstages; stage += 2) {
        load_frags(fb, stage + 1);
        compute(fa, stage);
        load_frags(fa, stage + 2);
        compute(fb, stage + 1);
    }
    float s = 0;
    for (int a = 0; a < TM; ++a) for (int b = 0; b < TN; ++b) for (int r = 0; r < 16; ++r) s += acc[a][b][r];
    out[blockIdx.x * NTH + tid] = s;
}

// mode 3: 16 x 16 x 32 MFMAs on register operands; per stage the same 16 x 32768 FLOP per wave as modes 0-2
template <int RANDOM>
__global__ __launch_bounds__(NTH) void probe16_kernel(float* out, int nstages)
{
    const int tid = threadIdx.x;
    f32x4 acc[16];
    for (int a = 0; a < 16; ++a) for (int r = 0; r < 4; ++r) acc[a][r] = 0.f;
    bf16x8 af[4], bfr[4];
    for (int i = 0; i < 4; ++i) {
        uint16_t va[8], vb[8];
        for (int e = 0; e < 8; ++e) {
            va[e] = RANDOM ? hash_bf16((tid * 8 + e) * 2654435761u + i * 977u + blockIdx.x) : (uint16_t)0x3c00;
            vb[e] = RANDOM ? hash_bf16((tid * 8 + e) * 40503u + i * 131u + 7u * blockIdx.x + 12345u) : (uint16_t)0x3c00;
        }
        __builtin_memcpy(&af[i], va, 16); __builtin_memcpy(&bfr[i], vb, 16);
    }
    for (int stage = 0; stage < nstages; ++stage) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)               // 2 x 16 MFMAs of 16 x 16 x 32 = 16 MFMAs of 32 x 32 x 16 in FLOP
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi * 4 + ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[mi], bfr[ni], acc[mi * 4 + ni], 0, 0, 0);
    }
    float s = 0;
    for (int a = 0; a < 16; ++a) for (int r = 0; r < 4; ++r) s += acc[a][r];
    out[blockIdx.x * NTH + tid] = s;
}

template <int MODE, int RANDOM>
static int run(const uint16_t* w, float* out, unsigned wbytes, double seconds)
{
    const int nstages = STAGES_PER_TILE * 8, nwg = 4096;
    const double flop = (double)nwg * nstages * MT * NT * KC * 2.0;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    auto launch = [&]() {
        if (MODE == 3) hipLaunchKernelGGL((probe16_kernel<RANDOM>), dim3(nwg), dim3(NTH), 0, 0, out, nstages);
        else if (MODE == 4) hipLaunchKernelGGL((probe_kernel<2, RANDOM, true>), dim3(nwg), dim3(NTH), 0, 0, w, out, nstages, wbytes);
        else if (MODE == 6) hipLaunchKernelGGL((probe_direct_kernel<RANDOM>), dim3(nwg), dim3(NTH), 0, 0, w, out, nstages, wbytes);
        else if (MODE == 5) hipLaunchKernelGGL((probe_kernel<2, RANDOM, false, 1>), dim3(nwg), dim3(NTH), 0, 0, w, out, nstages, wbytes);
        else hipLaunchKernelGGL((probe_kernel<(MODE >= 3 ? 0 : MODE), RANDOM>), dim3(nwg), dim3(NTH), 0, 0, w, out, nstages, wbytes);
    };
    launch();   // code load
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    launch();
    CK(hipEventRecord(e1)); CK(hipDeviceSynchronize());
    float first_ms; CK(hipEventElapsedTime(&first_ms, e0, e1));
    const int reps = (int)(seconds * 1e3 / first_ms) + 1;
    CK(hipEventRecord(e0));
    for (int r = 0; r < reps; ++r) launch();
    CK(hipEventRecord(e1)); CK(hipDeviceSynchronize());
    float total_ms; CK(hipEventElapsedTime(&total_ms, e0, e1));
    printf("mode %d random %d: first launch %.0f TFLOP/s; %d launches in %.0f ms: sustained %.0f TFLOP/s\n",
           MODE, RANDOM, flop / first_ms / 1e9, reps, total_ms, flop * reps / total_ms / 1e9);
    fflush(stdout);
    return 0;
}

int main(int argc, char** argv)
{
    const int mode = argc > 1 ? atoi(argv[1]) : 0;
    const double seconds = argc > 2 ? atof(argv[2]) : 3.0;
    const int random = argc > 3 ? atoi(argv[3]) : 1;
    if (mode < 0 || mode > 6 || seconds <= 0 || seconds > 30) {
        fprintf(stderr, "usage: mfma_probe <mode 0|1|2|3|4|5|6> <seconds (0, 30]> <random 0|1>\n");
        return 2;
    }
    const unsigned wbytes = (unsigned)N_TILES * STAGES_PER_TILE * MT * KC * 2;
    uint16_t* w; float* out;
    CK(hipMalloc(&w, wbytes)); CK(hipMalloc(&out, 4096 * NTH * sizeof(float)));
    uint16_t* hw = (uint16_t*)malloc(wbytes);
    unsigned x = 12345;
    for (unsigned i = 0; i < wbytes / 2; ++i) {
        x = x * 1664525u + 1013904223u;
        hw[i] = random ? (uint16_t)(((x >> 16) & 0x807f) | (0x3f00 + ((x >> 9) & 0x0080))) : (uint16_t)0x3c00;
    }
    CK(hipMemcpy(w, hw, wbytes, hipMemcpyHostToDevice));
    free(hw);
    int rc;
    if (random) rc = mode == 0 ? run<0, 1>(w, out, wbytes, seconds) : mode == 1 ? run<1, 1>(w, out, wbytes, seconds) : mode == 2 ? run<2, 1>(w, out, wbytes, seconds) : mode == 3 ? run<3, 1>(w, out, wbytes, seconds) : mode == 4 ? run<4, 1>(w, out, wbytes, seconds) : mode == 5 ? run<5, 1>(w, out, wbytes, seconds) : run<6, 1>(w, out, wbytes, seconds);
    else rc = mode == 0 ? run<0, 0>(w, out, wbytes, seconds) : mode == 1 ? run<1, 0>(w, out, wbytes, seconds) : mode == 2 ? run<2, 0>(w, out, wbytes, seconds) : mode == 3 ? run<3, 0>(w, out, wbytes, seconds) : mode == 4 ? run<4, 0>(w, out, wbytes, seconds) : mode == 5 ? run<5, 0>(w, out, wbytes, seconds) : run<6, 0>(w, out, wbytes, seconds);
    CK(hipFree(w)); CK(hipFree(out));
    return rc;
}
