// Sketch chain V_out = R * V_in (paper Section 4.2 and App. A.1: the products R(R(...(R S^T)))
// that make the fit cost O(n^2 p_s) instead of O(n^3)).  R is n x n fp32, V is n x p_s with the
// sketch width padded to ld = 16, 32 or 64 columns.  The product reads R exactly once and is bound
// by HBM bandwidth, so R never goes through LDS: every lane fetches 16 bytes of its row straight
// into registers and feeds v_mfma_f32_16x16x4_f32; only the small V is staged in LDS and shared by
// the four wavefronts of a workgroup.
//
//   workgroup = 4 wavefronts = 64 rows of R for one matrix, wave w owns rows 16w..16w+15
//   K runs in chunks of 64: lane (i = l % 16, q = l / 16) holds R[row i][k0 + 16 s + 4 q + e],
//   s = 0..3, e = 0..3; MFMA (s, e) pairs it with V[k0 + 16 s + 4 q + e][col] (the order of the
//   four k of one instruction is free as long as both operands agree).
//   V chunk in LDS: Vs[64][LD + 4]; with that stride the four lane groups of a fragment read
//   (rows 4 apart) fall on disjoint bank halves.
//   The loads of R run five chunks ahead of the MFMAs (the kernel is latency bound otherwise).
#include "common.h"

namespace prism {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int NT = 256;
constexpr int KC = 64;     // k per chunk
constexpr int ROWS = 64;   // rows of R per workgroup

template <int LD>
__global__ __launch_bounds__(NT, 2) void chain_kernel(const float* __restrict__ R, long long strideR, int ldr,
                                                   const float* __restrict__ Vin, long long strideVin,
                                                   float* __restrict__ Vout, long long strideVout, int n,
                                                   const Ctrl* __restrict__ ctrl) {
  constexpr int NBLK = LD / 16;
  constexpr int VS = LD + 4;
  __shared__ float Vs[2][KC][VS];
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int li = lane & 15, lq = lane >> 4;
  const int row0 = blockIdx.x * ROWS + wave * 16;
  const float* Rrow = R + (long long)b * strideR + (long long)(row0 + li) * ldr + 4 * lq;
  const float* Vb = Vin + (long long)b * strideVin;

  // V chunk loader: KC x LD floats = KC * LD / 4 float4, spread over the workgroup
  constexpr int V_LOADS = KC * LD / 4;
  constexpr int V_IT = (V_LOADS + NT - 1) / NT;
  f32x4 vreg[V_IT];
  auto load_v = [&](int k0) {
#pragma unroll
    for (int it = 0; it < V_IT; ++it) {
      const int idx = t + it * NT;
      if (V_LOADS % NT == 0 || idx < V_LOADS) {
        const int kr = idx / (LD / 4), c4 = idx % (LD / 4);
        vreg[it] = *(const f32x4*)(Vb + (long long)(k0 + kr) * LD + c4 * 4);
      }
    }
  };
  auto store_v = [&](int buf) {
#pragma unroll
    for (int it = 0; it < V_IT; ++it) {
      const int idx = t + it * NT;
      if (V_LOADS % NT == 0 || idx < V_LOADS) {
        const int kr = idx / (LD / 4), c4 = idx % (LD / 4);
        *(f32x4*)&Vs[buf][kr][c4 * 4] = vreg[it];
      }
    }
  };
  constexpr int DEPTH = 6;   // ring of chunks of this lane's row of R: loads run DEPTH-1 chunks ahead
  f32x4 ra[DEPTH][4];
  const int nchunks = n / KC;
  auto load_r = [&](int slot, int c) {   // slot is a compile-time constant at every call site
    if (c < nchunks) {
#pragma unroll
      for (int s = 0; s < 4; ++s) ra[slot][s] = *(const f32x4*)(Rrow + c * KC + 16 * s);
    }
  };

  f32x4 acc[NBLK];
#pragma unroll
  for (int j = 0; j < NBLK; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Workgroup barrier without the release fence of __syncthreads(): that fence waits for every
  // outstanding load and would expose the memory latency of the prefetched rows of R at every
  // chunk.  LDS traffic of this wave is complete (lgkmcnt(0)); loads into registers stay in flight.
  auto lds_barrier = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  load_v(0);
#pragma unroll
  for (int d = 0; d < DEPTH - 1; ++d) load_r(d, d);
  store_v(0);
  lds_barrier();
  for (int c0 = 0; c0 < nchunks; c0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int c = c0 + d;
      if (c < nchunks) {          // uniform
        const int cur = c & 1;
        // the small V chunk is requested before the rows of R further ahead, so that waiting for
        // it (to stage it in LDS) leaves those rows in flight
        if (c + 1 < nchunks) load_v((c + 1) * KC);
        load_r((d + DEPTH - 1) % DEPTH, c + DEPTH - 1);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int j = 0; j < NBLK; ++j)
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[d][s][e], Vs[cur][16 * s + 4 * lq + e][j * 16 + li], acc[j], 0, 0, 0);
        if (c + 1 < nchunks) store_v(cur ^ 1);
        lds_barrier();
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r)
      Vout[(long long)b * strideVout + (long long)(row0 + 4 * lq + r) * LD + j * 16 + li] = acc[j][r];
}

// Variant for small matrices (n <= 2048), where the kernel above is latency bound for lack of
// workgroups: a workgroup owns only 16 rows of R and its four wavefronts split K between them
// (wave w takes the chunks c = w, w+4, ...), each staging its own chunks of V in a private LDS
// area (no workgroup barrier inside the loop); the four partial sums are added through LDS in a
// fixed order at the end.
template <int LD>
__global__ __launch_bounds__(NT, 2) void chain_small_kernel(const float* __restrict__ R, long long strideR, int ldr,
                                                         const float* __restrict__ Vin, long long strideVin,
                                                         float* __restrict__ Vout, long long strideVout, int n,
                                                         const Ctrl* __restrict__ ctrl) {
  constexpr int NBLK = LD / 16;
  constexpr int VS = LD + 4;
  constexpr int VL = KC * LD / 4 / 64;          // float4 loads per lane for one chunk of V
  __shared__ float Vs[4][2][KC][VS];             // [wave][double buffer]
  __shared__ float red[4][NBLK][4][64];
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int li = lane & 15, lq = lane >> 4;
  const int row0 = blockIdx.x * 16;
  const float* Rrow = R + (long long)b * strideR + (long long)(row0 + li) * ldr + 4 * lq;
  const float* Vb = Vin + (long long)b * strideVin;
  const int nchunks = n / KC;
  const int mine = (nchunks - wave + 3) / 4;     // chunks of this wave

  constexpr int DEPTH = 3;
  f32x4 ra[DEPTH][4], va[DEPTH][VL];
  auto load = [&](int slot, int i) {             // i-th chunk of this wave; slot is compile time
    if (i < mine) {
      const int c = wave + 4 * i;
#pragma unroll
      for (int s = 0; s < 4; ++s) ra[slot][s] = *(const f32x4*)(Rrow + c * KC + 16 * s);
#pragma unroll
      for (int v = 0; v < VL; ++v) {
        const int idx = lane + 64 * v;
        va[slot][v] = *(const f32x4*)(Vb + (long long)(c * KC + idx / (LD / 4)) * LD + (idx % (LD / 4)) * 4);
      }
    }
  };
  f32x4 acc[NBLK];
#pragma unroll
  for (int j = 0; j < NBLK; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int d = 0; d < DEPTH - 1; ++d) load(d, d);
  for (int i0 = 0; i0 < mine; i0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int i = i0 + d;
      if (i < mine) {                             // uniform within the wave
        load((d + DEPTH - 1) % DEPTH, i + DEPTH - 1);
        const int buf = i & 1;
#pragma unroll
        for (int v = 0; v < VL; ++v) {
          const int idx = lane + 64 * v;
          *(f32x4*)&Vs[wave][buf][idx / (LD / 4)][(idx % (LD / 4)) * 4] = va[d][v];
        }
        // wave-private LDS area: LDS operations of one wave complete in order, no barrier needed
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int j = 0; j < NBLK; ++j)
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[d][s][e], Vs[wave][buf][16 * s + 4 * lq + e][j * 16 + li], acc[j], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][j][r][lane] = acc[j][r];
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int j = 0; j < NBLK; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = (red[0][j][r][lane] + red[1][j][r][lane]) + (red[2][j][r][lane] + red[3][j][r][lane]);
        Vout[(long long)b * strideVout + (long long)(row0 + 4 * lq + r) * LD + j * 16 + li] = v;
      }
  }
}

}  // namespace

// R: [batch][n][ldr] fp32 (n a multiple of 64), Vin/Vout: [n][ld] per matrix (strideVin may be 0)
int launch_chain(const float* R, long long strideR, int ldr, const float* Vin, long long strideVin, float* Vout,
                 long long strideVout, int n, int ld, int batch, const Ctrl* ctrl, hipStream_t s) {
  if (n % KC || n % ROWS || ldr % 4 || batch <= 0) return PRISM_EINVAL;
  // 64-row workgroups leave most CUs idle on small batches of small matrices: 16-row ones there
  if (ld <= 32 && (long long)(n / ROWS) * batch < 256) {
    const dim3 grid(n / 16, batch), block(NT);
    if (ld == 16) hipLaunchKernelGGL(chain_small_kernel<16>, grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
    else hipLaunchKernelGGL(chain_small_kernel<32>, grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
  }
  const dim3 grid(n / ROWS, batch), block(NT);
  if (ld == 16) hipLaunchKernelGGL(chain_kernel<16>, grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
  else if (ld == 32) hipLaunchKernelGGL(chain_kernel<32>, grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
  else if (ld == 64) hipLaunchKernelGGL(chain_kernel<64>, grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
  else return PRISM_EINVAL;
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

}  // namespace prism
