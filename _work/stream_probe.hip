// Measurement aid: the operand streams of the frozen-weight GEMM without any arithmetic.  Workgroup (tm, tn) pulls
// the 128 "A" rows of m-tile tm and the 128 "B" rows of n-tile tn, 128 bytes of every row per step, straight into an
// LDS ring with global_load_lds_dwordx4, with a chosen number of steps in flight and no barriers: the same addresses,
// the same sharing between workgroups (an A row is wanted by every n-tile, a B row by every m-tile) and the same
// workgroup-to-XCD mapping as gemm_nt_dl_kernel with 128x128 tiles.  What it reaches is the ceiling of that kernel's
// loads; the data is discarded.
#include "kernels.h"

template <int WAITN>
__global__ __launch_bounds__(256) void stream_probe_kernel(const char* __restrict__ A, const char* __restrict__ B,
                                                           unsigned ld, unsigned kbytes, int tiles_m, unsigned* sink) {
    __shared__ __align__(16) unsigned char lds[3 * 32768];
    int pid = blockIdx.x;
    const int nt = gridDim.x;
    if ((nt & 7) == 0) pid = (pid & 7) * (nt >> 3) + (pid >> 3);
    const int tm = pid % tiles_m, tn = pid / tiles_m;
    const unsigned wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    // wave w, load j: rows (w * 8 + j) * 8 + lane / 8 of the 256-row stack (A rows, then B rows), 16-byte chunk lane % 8
    unsigned voff[8];
    const char* base[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const unsigned r = (wave * 8 + j) * 8 + (lane >> 3);
        const bool is_a = r < 128;
        const unsigned row = is_a ? tm * 128 + r : tn * 128 + (r - 128);
        voff[j] = row * ld + (lane & 7) * 16;
        base[j] = is_a ? A : B;
    }
    const unsigned lbase = (unsigned)(size_t)lds + wave * 8192;
    unsigned slot = 0;
    for (unsigned k = 0; k < kbytes; k += 128) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const unsigned la = __builtin_amdgcn_readfirstlane(lbase + slot * 32768 + j * 1024);
            const char* b = base[j] + k;
            asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff[j]), "s"(b), "s"(la) : "memory");
        }
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(WAITN) : "memory");
        slot = slot == 2 ? 0 : slot + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (((unsigned*)lds)[threadIdx.x] == 0x9e3779b9u) *sink = 1;   // practically never: keeps the loads alive
}

// A: [tiles_m * 128 rows], B: [tiles_n * 128 rows], rows ld bytes apart, the first kbytes of each row are read.
hipError_t launch_stream_probe(const void* A, const void* B, unsigned ld, unsigned kbytes, int tiles_m, int tiles_n,
                               int steps_in_flight, unsigned* sink, hipStream_t s) {
    if (tiles_m <= 0 || tiles_n <= 0 || kbytes == 0 || (kbytes & 127) || kbytes > ld || (ld & 15)) return hipErrorInvalidValue;
    if ((size_t)tiles_m * 128 * ld >= (1ull << 32) || (size_t)tiles_n * 128 * ld >= (1ull << 32)) return hipErrorInvalidValue;
    const int grid = tiles_m * tiles_n;
#define TL_PROBE_GO(W) \
    stream_probe_kernel<W><<<grid, 256, 0, s>>>((const char*)A, (const char*)B, ld, kbytes, tiles_m, sink)
    switch (steps_in_flight) {
        case 1: TL_PROBE_GO(0); break;
        case 2: TL_PROBE_GO(8); break;
        case 3: TL_PROBE_GO(16); break;
        case 4: TL_PROBE_GO(24); break;
        case 6: TL_PROBE_GO(40); break;
        case 8: TL_PROBE_GO(56); break;
        default: return hipErrorInvalidValue;
    }
#undef TL_PROBE_GO
    return hipGetLastError();
}
