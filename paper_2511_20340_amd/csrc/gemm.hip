// Linear layers  y[M][N] = x[M][K] . w[N][K]^T (+bias) (+residual)  for gfx950.
//
// bf16 path ("weight-direct").  Decoding GEMMs are skinny: M = B*(k+1) rows against weight
// matrices that are streamed from HBM exactly once.  The weights are therefore kept PACKED in
// MFMA-operand order (pack_weight below): for every 32-row block of W and every 16-wide k-step
// one 1 KiB unit holds, lane by lane, the 8 bf16 a lane feeds to v_mfma_f32_32x32x16_bf16.  A
// wavefront owns TN such row blocks and streams them straight from global memory into operand
// registers with fully coalesced 16-byte loads -- no LDS traffic, no barrier on the weight side.
// Only the activations (BM = TM*32 rows x 64 k) are staged through LDS (register-prefetched
// double buffer, rows padded to 72 elements: conflict-free 16-byte operand reads) and shared by
// the 4 waves of the workgroup, which cover 4*TN*32 output columns.
//
// Parallelism for small N*M: the K dimension is split over `split_k` workgroups per tile.  Each
// leaves its fp32 partial tile in the workspace and takes a ticket; the last one to arrive adds
// the partials in split order (deterministic), applies the epilogue and resets the ticket, so one
// launch does everything and the counters stay zero between launches.
//
// Workgroup ids are remapped so that all M-tiles of one weight column block run on the same XCD
// (its L2 then serves the weight units to every M-tile after one HBM read).
//
// fp32 path: plain SIMT tiling on row-major weights for the small fp32 configuration.
#include "sf_internal.h"

namespace sf {
namespace {

constexpr int BK = 64;
constexpr int LDK = 72;  // padded LDS row length in bf16 elements (144 B)
constexpr int XCDS = 8;

template <int TM, int TN, int OCC>
__global__ __launch_bounds__(256, OCC) void gemm_wd_kernel(const bf16_t *__restrict__ A, const uint4 *__restrict__ Wp,
                                                      const bf16_t *__restrict__ bias, const bf16_t *residual,
                                                      void *Y, int M, int N, int K, int out_f32, int tiles_m,
                                                      int tiles_n, int split_k, int kt_per_split,
                                                      float *__restrict__ partial, unsigned *__restrict__ tickets,
                                                      int glu) {
  constexpr int BM = TM * 32;
  extern __shared__ __attribute__((aligned(16))) bf16_t sA[];  // [2][BM][LDK]
  __shared__ unsigned s_ticket;

  // XCD-aware tile assignment: consecutive workgroup ids round-robin over the 8 XCDs; inside an
  // XCD the M-tiles of a column block are adjacent, then the K splits, then the next column block.
  const int id = blockIdx.x;
  const int xcd = id % XCDS, j = id / XCDS;
  const int tm = j % tiles_m, ks = (j / tiles_m) % split_k;
  const int tn = (j / (tiles_m * split_k)) * XCDS + xcd;
  if (tn >= tiles_n) return;
  const int m0 = tm * BM;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int n_blocks = (N + 31) >> 5;        // 32-row blocks of W
  const int k_steps = (K + 15) >> 4;         // 16-wide k-steps (packed K is padded to 16)
  const int nb0 = (tn * 4 + wave) * TN;      // this wave's first W row block

  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  uint4 ra[TM];                    // activation chunks in flight to LDS
  uint4 wcur[4][TN], wnxt[4][TN];  // weight operands of the current / next K slice
  auto aload = [&](int k0) {
#pragma unroll
    for (int c = 0; c < TM; ++c) {
      const int cid = tid + 256 * c, row = cid >> 3, kc = (cid & 7) * 8;
      const int gr = m0 + row;
      ra[c] = (gr < M && k0 + kc < K) ? *reinterpret_cast<const uint4 *>(A + (size_t)gr * K + k0 + kc)
                                      : make_uint4(0, 0, 0, 0);
    }
  };
  auto astore = [&](int buf) {
#pragma unroll
    for (int c = 0; c < TM; ++c) {
      const int cid = tid + 256 * c, row = cid >> 3, kc = (cid & 7) * 8;
      *reinterpret_cast<uint4 *>(sA + (buf * BM + row) * LDK + kc) = ra[c];
    }
  };
  auto wload = [&](uint4 (&w)[4][TN], int kt) {
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int b = 0; b < TN; ++b) {
        const int kstep = kt * 4 + s, nb = nb0 + b;
        w[s][b] = (kstep < k_steps && nb < n_blocks) ? Wp[((size_t)nb * k_steps + kstep) * 64 + lane]
                                                     : make_uint4(0, 0, 0, 0);
      }
  };

  const int KT = (K + BK - 1) / BK;
  const int kt0 = ks * kt_per_split, kt1 = min(KT, kt0 + kt_per_split);
  if (kt0 < kt1) {
    wload(wcur, kt0);
    aload(kt0 * BK);
    astore(0);
  }
  __syncthreads();
  for (int kt = kt0; kt < kt1; ++kt) {
    const int buf = (kt - kt0) & 1;
    const bool more = kt + 1 < kt1;
    if (more) {
      wload(wnxt, kt + 1);
      aload((kt + 1) * BK);
    }
    const bf16_t *pa = sA + (buf * BM + ln) * LDK + lh * 8;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        const bf16x8 fa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pa + a * 32 * LDK + s * 16));
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, __builtin_bit_cast(bf16x8, wcur[s][b]), acc[a][b],
                                                              0, 0, 0);
      }
    }
    if (more) {
      astore(buf ^ 1);
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int b = 0; b < TN; ++b) wcur[s][b] = wnxt[s][b];
    }
    __syncthreads();
  }

  if (split_k > 1) {
    // Partial tiles in register order: [tile][split][wave][TM][TN][reg][lane].  They are written
    // and read with agent-scope accesses (write-through / cache-bypassing), so no L2-wide
    // writeback or invalidate is needed to make them visible to the workgroup that finishes.
    const size_t tile = (size_t)tn * tiles_m + tm;
    constexpr size_t PER_WAVE = (size_t)TM * TN * 64 * 16;
    float *mine = partial + ((tile * split_k + ks) * 4 + wave) * PER_WAVE;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          __hip_atomic_store(mine + ((a * TN + b) * 16 + v) * 64 + lane, acc[a][b][v], __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // this wave's stores have been acknowledged
    __syncthreads();
    if (tid == 0) s_ticket = __hip_atomic_fetch_add(&tickets[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != (unsigned)(split_k - 1)) return;  // not the last split of this tile
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    for (int s = 0; s < split_k; ++s) {  // fixed order: the sum does not depend on arrival order
      const float *p = partial + ((tile * split_k + s) * 4 + wave) * PER_WAVE;
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            acc[a][b][v] += __hip_atomic_load(p + ((a * TN + b) * 16 + v) * 64 + lane, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid == 0) __hip_atomic_store(&tickets[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  if (glu) {
    // SwiGLU epilogue.  The weight was packed with gate and up rows interleaved 16 by 16, so a
    // 32-column tile holds gate features f..f+15 in columns 0-15 and the matching up features in
    // columns 16-31: lane ln < 16 fetches its partner's value and writes silu(gate) * up.
    const int F = N >> 1;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b) {
        const int col = (nb0 + b) * 16 + (ln & 15);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float mine = acc[a][b][v];
          const float other = __shfl_xor(mine, 16);
          const int row = m0 + a * 32 + c_row(v, lh);
          if ((ln & 16) == 0 && col < F && row < M) {
            const float r = mine / (1.0f + __expf(-mine)) * other;
            reinterpret_cast<bf16_t *>(Y)[(size_t)row * F + col] = f2bf(r);
          }
        }
      }
    return;
  }

  // epilogue: lane holds column ln, rows c_row(v, lh) of every 32x32 tile
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int col = (nb0 + b) * 32 + ln;
      if (col >= N) continue;
      const float bv = bias ? bf2f(bias[col]) : 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + a * 32 + c_row(v, lh);
        if (row >= M) continue;
        float r = acc[a][b][v] + bv;
        const size_t o = (size_t)row * N + col;
        if (residual) r += bf2f(residual[o]);
        if (out_f32) reinterpret_cast<float *>(Y)[o] = r;
        else reinterpret_cast<bf16_t *>(Y)[o] = f2bf(r);
      }
    }
}

// row-major [N][K] -> packed units; one thread per 16-byte operand register
// glu_F > 0: W is [2F][K] = [gate; up] and packed row block nb holds gate rows 16nb..16nb+15 followed
// by up rows 16nb..16nb+15 (see the SwiGLU epilogue)
__global__ void pack_weight_kernel(const bf16_t *__restrict__ W, uint4 *__restrict__ P, int N, int K, size_t units,
                                   int glu_F) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= units) return;
  const int lane = idx & 63;
  const size_t u = idx >> 6;
  const int k_steps = (K + 15) >> 4;
  const int kstep = u % k_steps;
  const int nb = u / k_steps;
  int row = nb * 32 + (lane & 31);
  const int k0 = kstep * 16 + (lane >> 5) * 8;
  if (glu_F > 0) {
    const int within = lane & 31, f = nb * 16 + (within & 15);
    row = f < glu_F ? (within < 16 ? f : glu_F + f) : N;
  }
  uint32_t w[4] = {0, 0, 0, 0};
  if (row < N)
    for (int e = 0; e < 8; ++e)
      if (k0 + e < K) w[e >> 1] |= (uint32_t)W[(size_t)row * K + k0 + e] << ((e & 1) * 16);
  P[idx] = make_uint4(w[0], w[1], w[2], w[3]);
}

struct Plan {
  int tiles_m, tiles_n, split_k, kt_per_split;
  size_t partial_bytes, ticket_bytes;
};

// The split factor depends on the weight shape only (never on M), so a row's result is
// bit-identical whatever else is batched with it: ~256 workgroups per M-tile, at least 8 K slices
// (512 of K) per split.  Shapes with enough column tiles are not split.
int auto_split(int N, int K) {
  const int KT = (K + BK - 1) / BK;
  const int col_tiles = (N + 127) / 128;
  int s = 1;
  while (s * 2 * col_tiles <= 256 && KT / (s * 2) >= 8 && s < 16) s *= 2;
  return s;
}

Plan make_plan(int M, int N, int K, int BM, int BN, int split_req) {
  Plan p;
  p.tiles_m = (M + BM - 1) / BM;
  p.tiles_n = (N + BN - 1) / BN;
  const int KT = (K + BK - 1) / BK;
  const int tiles = p.tiles_m * p.tiles_n;
  int s = split_req > 0 ? split_req : (M <= 640 ? auto_split(N, K) : 1);
  s = s < 1 ? 1 : (s > KT ? KT : s);
  p.kt_per_split = (KT + s - 1) / s;
  p.split_k = (KT + p.kt_per_split - 1) / p.kt_per_split;
  p.partial_bytes = p.split_k > 1 ? (size_t)tiles * p.split_k * BM * BN * sizeof(float) : 0;
  p.ticket_bytes = p.split_k > 1 ? (size_t)tiles * sizeof(unsigned) : 0;
  return p;
}

template <int TM, int TN, int OCC>
hipError_t run_wd(const GemmArgs &a, hipStream_t s, int split_req) {
  constexpr int BM = TM * 32, BN = 4 * TN * 32;
  Plan p = make_plan(a.M, a.N, a.K, BM, BN, split_req);
  if (p.split_k > 1 && (!a.ws || a.ws_bytes < GEMM_TICKET_BYTES + p.partial_bytes ||
                        p.ticket_bytes > GEMM_TICKET_BYTES)) {
    p = make_plan(a.M, a.N, a.K, BM, BN, 1);  // no room for partials: single pass
  }
  const int groups = (p.tiles_n + XCDS - 1) / XCDS;
  const size_t lds = (size_t)2 * BM * LDK * sizeof(bf16_t);
  auto kern = gemm_wd_kernel<TM, TN, OCC>;
  static bool attr_done = false;
  if (!attr_done && lds > 48 * 1024) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    attr_done = true;
  }
  unsigned *tickets = (unsigned *)a.ws;
  float *partial = a.ws ? (float *)((char *)a.ws + GEMM_TICKET_BYTES) : nullptr;
  kern<<<dim3(groups * XCDS * p.tiles_m * p.split_k), dim3(256), lds, s>>>(
      (const bf16_t *)a.x, (const uint4 *)a.w, (const bf16_t *)a.bias, (const bf16_t *)a.residual, a.y, a.M, a.N,
      a.K, a.out_f32, p.tiles_m, p.tiles_n, p.split_k, p.kt_per_split, partial, tickets, a.glu);
  return hipGetLastError();
}

// fp32: 64x64 tile, 16 wide k slices, each thread a 4x4 micro-tile
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ W,
                                                       const float *__restrict__ bias, const float *residual,
                                                       float *Y, int M, int N, int K) {
  __shared__ float sA[16][65], sW[16][65];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int x = tid; x < 64 * 16; x += 256) {
      const int r = x >> 4, kk = x & 15;
      sA[kk][r] = (m0 + r < M && k0 + kk < K) ? A[(size_t)(m0 + r) * K + k0 + kk] : 0.f;
      sW[kk][r] = (n0 + r < N && k0 + kk < K) ? W[(size_t)(n0 + r) * K + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = sA[kk][ty * 4 + i]; wv[i] = sW[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) acc[i][jn] += av[i] * wv[jn];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) {
      const int r = m0 + ty * 4 + i, c = n0 + tx * 4 + jn;
      if (r < M && c < N) {
        float v = acc[i][jn] + (bias ? bias[c] : 0.f);
        if (residual) v += residual[(size_t)r * N + c];
        Y[(size_t)r * N + c] = v;
      }
    }
}

int g_tile = 0, g_split = 0;  // tuning overrides (0 = automatic)

}  // namespace

void gemm_tune(int tile, int split_k) { g_tile = tile; g_split = split_k; }

size_t gemm_workspace_bytes(int M_max) {
  (void)M_max;
  return GEMM_TICKET_BYTES + GEMM_PARTIAL_BYTES;
}

size_t packed_weight_bytes(int N, int K, int dtype) {
  if (dtype != SF_BF16) return (size_t)N * K * sizeof(float);
  return (size_t)((N + 31) / 32) * ((K + 15) / 16) * 1024;
}

hipError_t launch_pack_weight(const void *w, void *packed, int N, int K, int glu, int dtype, hipStream_t s) {
  if (dtype != SF_BF16) return hipMemcpyAsync(packed, w, (size_t)N * K * sizeof(float), hipMemcpyDeviceToDevice, s);
  const size_t units = packed_weight_bytes(N, K, dtype) / 16;
  pack_weight_kernel<<<(unsigned)((units + 255) / 256), 256, 0, s>>>((const bf16_t *)w, (uint4 *)packed, N, K, units,
                                                                     glu ? N / 2 : 0);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16(const GemmArgs &a, hipStream_t s) {
  int tile = g_tile;
  if (tile == 0) {
    // Rows per workgroup.  Small weight matrices stay resident in L2 / the last-level cache, so
    // re-reading them for every 32- or 64-row M-tile is cheap and the many small workgroups hide
    // the per-slice latency better; large ones are streamed once per 160 (or 128) rows.
    const size_t wbytes = (size_t)a.N * a.K * 2;
    const size_t MB = 1u << 20;
    if (a.M <= 32 || wbytes <= 40 * MB) tile = 1;
    else if (a.M <= 64 || wbytes <= 64 * MB || (a.M <= 160 && wbytes <= 160 * MB)) tile = 2;
    else if (a.M <= 128) tile = 3;
    else if (a.M <= 160 || a.M % 160 == 0) tile = 5;
    else if (a.M % 128 == 0 && a.M <= 512 && a.N >= 65536) tile = 4;
    else tile = 3;
  }
  switch (tile) {
    case 1: return run_wd<1, 1, 4>(a, s, g_split);
    case 2: return run_wd<2, 1, 4>(a, s, g_split);
    case 3: return run_wd<4, 1, 3>(a, s, g_split);
    case 4: return run_wd<4, 2, 2>(a, s, g_split);
    case 5: return run_wd<5, 1, 3>(a, s, g_split);
    case 6: return run_wd<5, 2, 1>(a, s, g_split);
    case 7: return run_wd<2, 2, 3>(a, s, g_split);
    default: return run_wd<4, 1, 3>(a, s, g_split);
  }
}

hipError_t launch_gemm_f32(const GemmArgs &a, hipStream_t s) {
  dim3 grid((a.N + 63) / 64, (a.M + 63) / 64);
  gemm_f32_kernel<<<grid, 256, 0, s>>>((const float *)a.x, (const float *)a.w, (const float *)a.bias,
                                       (const float *)a.residual, (float *)a.y, a.M, a.N, a.K);
  return hipGetLastError();
}

}  // namespace sf
