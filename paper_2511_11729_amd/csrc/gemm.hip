// 16-bit (half or bf16 operands, fp32 accumulate) MFMA GEMM for gfx950 (the compute-bound half of the co-located pair: Harli Sec. 1 /
// Sec. 2.1 -- PEFT finetuning is dominated by frozen-base matrix multiplications).
//
// Workgroup tile 256 x 128, K step 64, 4 waves in a 2 x 2 arrangement, each wave a 128 x 64
// tile = 4 x 2 v_mfma_f32_32x32x16_bf16 accumulators (128 fp32 registers per lane).
// Operands go global -> registers -> LDS (row-major rows of 64 k padded to 144 bytes, which
// makes both the 16-byte row writes and the 32-row fragment reads bank-conflict free) with
// two LDS stages and one barrier per K step.  Tiles are handed to XCDs in contiguous runs so
// that the workgroups sharing an L2 also share operand panels.
#include "gemm.h"

#include <vector>

#include "ctx.h"
#include "device_utils.h"

namespace harli {
namespace {

constexpr int BM = 256, BN = 128, BK = 64;
constexpr int ROWB = BK * 2 + 16;  // bytes per staged row
constexpr int A_STAGE = BM * ROWB, B_STAGE = BN * ROWB, STAGE = A_STAGE + B_STAGE;
constexpr int LDS_BYTES = 2 * STAGE;
constexpr int A_CH = BM * (BK / 8) / 256, B_CH = BN * (BK / 8) / 256;  // 16-byte chunks per thread per stage

struct StageCursor {
  int seg, k0, kend;
};

__device__ __forceinline__ void seg_range(const GemmArgs& a, int s, int m0, int* kb, int* ke) {
  const int K = a.seg[s].K;
  *kb = (a.causal == GEMM_K_FROM_M) ? (m0 / BK) * BK : 0;
  *ke = (a.causal == GEMM_K_UPTO_M) ? min(K, m0 + BM) : K;
}

template <bool HALF>
__global__ void __launch_bounds__(256) k_gemm(GemmArgs a, int tiles_n, int tiles_total, int chunk) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // XCD-aware tile order: workgroup w runs on XCD w % 8; give each XCD a contiguous run of tiles
  const int w = blockIdx.x;
  const int tile = (w & 7) * chunk + (w >> 3);
  if (tile >= tiles_total) return;
  const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  if (a.causal == GEMM_OUT_LOWER && n0 > m0 + BM - 1) return;
  if (a.causal == GEMM_OUT_UPPER && n0 + BN - 1 < m0) return;
  const int z = blockIdx.z, z2 = z % a.nb2, zq = z / a.nb2, z1 = zq % a.nb1, z0 = zq / a.nb1;

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // per-thread chunk coordinates (same for every stage)
  const int crow = tid >> 3, ckc = (tid & 7) * 8;
  uint4 ra[A_CH], rb[B_CH];

  StageCursor cur;
  cur.seg = 0;
  seg_range(a, 0, m0, &cur.k0, &cur.kend);
  while (cur.seg < a.nseg && cur.k0 >= cur.kend) {  // skip empty segments
    ++cur.seg;
    if (cur.seg < a.nseg) seg_range(a, cur.seg, m0, &cur.k0, &cur.kend);
  }

  auto fetch = [&](const StageCursor& c) {
    const GemmSeg& sg = a.seg[c.seg];
    const unsigned short* A = sg.A + z0 * sg.a_bs0 + z1 * sg.a_bs1 + z2 * sg.a_bs2;
    const unsigned short* B = sg.B + z0 * sg.b_bs0 + z1 * sg.b_bs1 + z2 * sg.b_bs2;
    const int k = c.k0 + ckc;
    const bool kok = k < sg.K;
    const int kc = kok ? k : sg.K - 8;  // clamp: every load stays in bounds, tails are zeroed below
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int r = m0 + crow + i * 32;
      const int rc = r < a.M ? r : a.M - 1;
      ra[i] = *reinterpret_cast<const uint4*>(A + (long long)rc * sg.lda + kc);
      if (!kok || r >= a.M) ra[i] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int r = n0 + crow + i * 32;
      const int rc = r < a.N ? r : a.N - 1;
      rb[i] = *reinterpret_cast<const uint4*>(B + (long long)rc * sg.ldb + kc);
      if (!kok || r >= a.N) rb[i] = make_uint4(0, 0, 0, 0);
    }
  };
  auto stash = [&](int buf) {
    char* sa = smem + buf * STAGE;
    char* sb = sa + A_STAGE;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<uint4*>(sa + (crow + i * 32) * ROWB + ckc * 2) = ra[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<uint4*>(sb + (crow + i * 32) * ROWB + ckc * 2) = rb[i];
  };
  auto advance = [&](StageCursor& c) {
    c.k0 += BK;
    while (c.seg < a.nseg && c.k0 >= c.kend) {
      ++c.seg;
      if (c.seg < a.nseg) seg_range(a, c.seg, m0, &c.k0, &c.kend);
    }
  };

  if (cur.seg < a.nseg) {
    fetch(cur);
    stash(0);
    advance(cur);
  }
  __syncthreads();
  int buf = 0;
  bool more = true;
  while (more) {
    const bool have_next = cur.seg < a.nseg;
    if (have_next) fetch(cur);
    const char* sa = smem + buf * STAGE + (wm * 128 + (lane & 31)) * ROWB + (lane >> 5) * 16;
    const char* sb = smem + buf * STAGE + A_STAGE + (wn * 64 + (lane & 31)) * ROWB + (lane >> 5) * 16;
#pragma unroll
    for (int sub = 0; sub < BK / 16; ++sub) {
      uint4 fa[4], fb[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const uint4*>(sa + i * 32 * ROWB + sub * 32);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const uint4*>(sb + j * 32 * ROWB + sub * 32);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = HALF ? __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fa[i]),
                                                                    __builtin_bit_cast(f16x8, fb[j]), acc[i][j], 0, 0, 0)
                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),
                                                                     __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
    }
    if (have_next) {
      stash(buf ^ 1);
      advance(cur);
    }
    more = have_next;
    buf ^= 1;
    __syncthreads();
  }

  // ---- epilogue: lane holds rows 8*(v/4) + 4*(lane/32) + v%4 of column lane%32 of each 32x32 tile ----
  const int col_l = lane & 31, rgrp = (lane >> 5) * 4;
  unsigned short* Cb = a.Cb ? a.Cb + z0 * a.cb_bs0 + z1 * a.cb_bs1 + z2 * a.cb_bs2 : nullptr;
  float* Cf = a.Cf ? a.Cf + z0 * a.cf_bs0 + z1 * a.cf_bs1 + z2 * a.cf_bs2 : nullptr;
  const float* Rs = a.res ? a.res + z0 * a.cf_bs0 + z1 * a.cf_bs1 + z2 * a.cf_bs2 : nullptr;
  unsigned short* Ct = a.Ct ? a.Ct + z0 * a.ct_bs0 + z1 * a.ct_bs1 + z2 * a.ct_bs2 : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn * 64 + j * 32 + col_l;
      if (n >= a.N) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int mb = m0 + wm * 128 + i * 32 + q * 8 + rgrp;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[e] = acc[i][j][q * 4 + e] * a.alpha;
          const int m = mb + e;
          if (m < a.M) {
            if (Cf) {
              const float r = Rs ? Rs[(long long)m * a.ldcf + n] : 0.f;
              o[e] += r;
              Cf[(long long)m * a.ldcf + n] = o[e];
            }
            if (Cb) Cb[(long long)m * a.ldcb + n] = HALF ? f2h(o[e]) : f2bf(o[e]);
          }
        }
        if (Ct) {
          unsigned short* p = Ct + (long long)n * a.ldct + mb;
          if (mb + 3 < a.M && ((a.ldct & 3) == 0)) {
            *reinterpret_cast<uint2*>(p) = HALF ? make_uint2(pack_h2(o[0], o[1]), pack_h2(o[2], o[3]))
                                                : make_uint2(pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3]));
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (mb + e < a.M) p[e] = HALF ? f2h(o[e]) : f2bf(o[e]);
          }
        }
      }
    }
}

}  // namespace

// ---- optional per-launch timing (harli_prof_*): two events around every GEMM launch ----
namespace {
struct ProfRec {
  hipEvent_t e0, e1;
  double flops;
};
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
}  // namespace

void gemm_prof_enable(bool on) { g_prof_on = on; }

harli_status gemm_prof_collect(double* flops, double* ms, long long* launches) {
  double f = 0.0, t = 0.0;
  for (ProfRec& r : g_prof) {
    HARLI_HIP(hipEventSynchronize(r.e1));
    float dt = 0.f;
    HARLI_HIP(hipEventElapsedTime(&dt, r.e0, r.e1));
    f += r.flops;
    t += dt;
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  *flops = f;
  *ms = t;
  *launches = (long long)g_prof.size();
  g_prof.clear();
  return HARLI_OK;
}

// flops the launch is asked to perform: full products for GEMM_FULL, the causal half otherwise
static double gemm_flops(const GemmArgs& a, int batches) {
  double k = 0;
  for (int s = 0; s < a.nseg; ++s) k += a.seg[s].K;
  const double f = 2.0 * a.M * (double)a.N * k * batches;
  return a.causal == GEMM_FULL ? f : 0.5 * f;
}

harli_status gemm_launch(const GemmArgs& a, int batches, hipStream_t st) {
  if (a.M < 1 || a.N < 1 || a.nseg < 1 || a.nseg > kGemmMaxSeg || batches < 1 || a.nb1 < 1 || a.nb2 < 1)
    return fail(HARLI_ERR_INVALID, "gemm: bad shape M %d N %d nseg %d batches %d", a.M, a.N, a.nseg, batches);
  for (int s = 0; s < a.nseg; ++s) {
    const GemmSeg& g = a.seg[s];
    if (!g.A || !g.B || g.K < 8 || (g.K & 7) || (g.lda & 7) || (g.ldb & 7) || (g.a_bs0 & 7) || (g.a_bs1 & 7) || (g.a_bs2 & 7) ||
        (g.b_bs0 & 7) || (g.b_bs1 & 7) || (g.b_bs2 & 7) || ((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15))
      return fail(HARLI_ERR_INVALID, "gemm: segment %d needs K %% 8 == 0 and 16-byte aligned rows (K %d lda %lld ldb %lld)", s,
                  g.K, g.lda, g.ldb);
  }
  if (!a.Cb && !a.Cf && !a.Ct) return fail(HARLI_ERR_INVALID, "gemm: no output");
  if (a.res && !a.Cf) return fail(HARLI_ERR_INVALID, "gemm: a residual needs the fp32 output");
  static bool attr_set = false;
  if (!attr_set) {
    HARLI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<true>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
    HARLI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<false>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
    attr_set = true;
  }
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n, chunk = (total + 7) / 8;
  ProfRec rec{};
  if (g_prof_on) {
    HARLI_HIP(hipEventCreate(&rec.e0));
    HARLI_HIP(hipEventCreate(&rec.e1));
    rec.flops = gemm_flops(a, batches);
    HARLI_HIP(hipEventRecord(rec.e0, st));
  }
  if (a.half)
    hipLaunchKernelGGL(k_gemm<true>, dim3(chunk * 8, 1, batches), dim3(256), LDS_BYTES, st, a, tiles_n, total, chunk);
  else
    hipLaunchKernelGGL(k_gemm<false>, dim3(chunk * 8, 1, batches), dim3(256), LDS_BYTES, st, a, tiles_n, total, chunk);
  if (g_prof_on) {
    HARLI_HIP(hipEventRecord(rec.e1, st));
    g_prof.push_back(rec);
  }
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}

}  // namespace harli
