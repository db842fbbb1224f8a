// 16-bit (half or bf16 operands, fp32 accumulate) MFMA GEMM for gfx950 (the compute-bound half of the co-located pair: Harli Sec. 1 /
// Sec. 2.1 -- PEFT finetuning is dominated by frozen-base matrix multiplications).
//
// Workgroup tile 256 x 128, K step 64, 8 waves in a 4 x 2 arrangement, each wave a 64 x 64
// tile = 2 x 2 v_mfma_f32_32x32x16 accumulators (64 fp32 registers per lane).
// Operands go global -> registers -> LDS (row-major rows of 64 k padded to 144 bytes, which
// makes both the 16-byte row writes and the 32-row fragment reads bank-conflict free) with
// two LDS stages and one barrier per K step.  Tiles are handed to XCDs in contiguous runs of
// 4 x 8-tile blocks so that the workgroups sharing an L2 also share operand panels.
#include "gemm.h"

#include <algorithm>
#include <vector>

#include "ctx.h"
#include "device_utils.h"

namespace harli {
namespace {

constexpr int BM = 256, BN = 128, BK = 64;
constexpr int kGM = 4, kGN = 8;  // tiles per L2-sharing block (clipped to the tile grid)
constexpr int ROWB = BK * 2 + 16;  // bytes per staged row
constexpr int A_STAGE = BM * ROWB, B_STAGE = BN * ROWB, STAGE = A_STAGE + B_STAGE;
constexpr int LDS_BYTES = 2 * STAGE;
constexpr int NT = 512;  // 8 waves, two per SIMD
constexpr int A_CH = BM * (BK / 8) / NT, B_CH = BN * (BK / 8) / NT;  // 16-byte chunks per thread per stage

__device__ __forceinline__ void seg_range(const GemmArgs& a, int s, int m0, int* kb, int* ke) {
  const int K = a.seg[s].K;
  *kb = (a.causal == GEMM_K_FROM_M) ? (m0 / BK) * BK : 0;
  *ke = (a.causal == GEMM_K_UPTO_M) ? min(K, m0 + BM) : K;
}

// One workgroup of 8 waves per CU, two waves per SIMD (256 registers each): while one wave of a SIMD waits on its
// staging loads, LDS writes or the barrier, the other one issues MFMAs.  (Four waves with twice the tile each and
// the whole register file were 27 % slower: nothing covered those waits.)
template <bool HALF, int EPI>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) k_gemm(GemmArgs a, int tiles_n, int tiles_total, int chunk, int GM, int GN, const uint4* zero16) {
  extern __shared__ __align__(16) char smem[];
  // Instruction-issue priority of these waves over the neighbour's (the co-located decode kernels wait on memory most
  // of the time and have slack under their latency target): about 1 % more finetune throughput beside decode, nothing alone.
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;  // 4 x 2 waves of 64 x 64
  // XCD-aware tile order: workgroup w runs on XCD w % 8.  Each XCD gets a contiguous run of slots, and slots
  // walk the tile grid in blocks of GM x GN tiles, so the 32 workgroups resident on an XCD at a time share
  // GM row panels of A and GN row panels of B in its L2 (4 + 8 panels instead of 1 + 32 for a row of tiles).
  const int w = blockIdx.x;
  const int slot = (w & 7) * chunk + (w >> 3);
  if (slot >= tiles_total) return;
  const int nbn = (tiles_n + GN - 1) / GN;
  const int blk = slot / (GM * GN), within = slot - blk * (GM * GN);
  const int bm = blk / nbn, bn = blk - bm * nbn;
  const int tm = bm * GM + within / GN, tn = bn * GN + within % GN;
  const int m0 = tm * BM, n0 = tn * BN;
  if (m0 >= a.M || n0 >= a.N) return;
  if (a.causal == GEMM_OUT_LOWER && n0 > m0 + BM - 1) return;
  if (a.causal == GEMM_OUT_UPPER && n0 + BN - 1 < m0) return;
  const int z = blockIdx.z, z2 = z % a.nb2, zq = z / a.nb2, z1 = zq % a.nb1, z0 = zq / a.nb1;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // per-thread chunk coordinates (same for every stage)
  const int crow = tid >> 3, ckc = (tid & 7) * 8;
  // Two register stages (sets r and q) are in flight besides the two LDS stages: a stage's global
  // loads are issued two compute phases before they are written to LDS.
  // They are named scalars, not arrays: the arrays were left in scratch memory by the compiler.
  static_assert(A_CH == 4 && B_CH == 2, "the staging macros below are written for 4 + 2 chunks per thread");
  uint4 ra0, ra1, ra2, ra3, rb0, rb1;
  uint4 qa0, qa1, qa2, qa3, qb0, qb1;
  // Row pointers of the current K segment live in registers and advance by BK per stage, so a
  // stage's loads need no address arithmetic beyond one select: out-of-range chunks (rows past
  // M / N, k past the segment) read a zero word instead -- selecting the ADDRESS keeps every
  // load unconditional (zeroing the loaded register made the compiler wait for each load in turn).
  const unsigned short* pa[A_CH];
  const unsigned short* pb[B_CH];
  bool oka[A_CH], okb[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) oka[i] = m0 + crow + i * 64 < a.M;
#pragma unroll
  for (int i = 0; i < B_CH; ++i) okb[i] = n0 + crow + i * 64 < a.N;
  int seg = -1, k0 = 0, kend = 0, Kseg = 0;

  // (written out with macros rather than lambdas: arrays captured by reference ended up in scratch)
#define OPEN_SEG(found)                                                                                   \
  do {                                                                                                    \
    for (++seg; seg < a.nseg; ++seg) {                                                                    \
      seg_range(a, seg, m0, &k0, &kend);                                                                  \
      if (k0 < kend) break;                                                                               \
    }                                                                                                     \
    (found) = seg < a.nseg;                                                                               \
    if (found) {                                                                                          \
      const GemmSeg& sg = a.seg[seg];                                                                     \
      Kseg = sg.K;                                                                                        \
      const unsigned short* A_ = sg.A + z0 * sg.a_bs0 + z1 * sg.a_bs1 + z2 * sg.a_bs2;                    \
      const unsigned short* B_ = sg.B + z0 * sg.b_bs0 + z1 * sg.b_bs1 + z2 * sg.b_bs2;                    \
      _Pragma("unroll") for (int i = 0; i < A_CH; ++i)                                                    \
          pa[i] = A_ + (long long)(m0 + crow + i * 64) * sg.lda + k0 + ckc;                               \
      _Pragma("unroll") for (int i = 0; i < B_CH; ++i)                                                    \
          pb[i] = B_ + (long long)(n0 + crow + i * 64) * sg.ldb + k0 + ckc;                               \
    }                                                                                                     \
  } while (0)
#define LDA_(S, i) S##a##i = *((kok && oka[i]) ? reinterpret_cast<const uint4*>(pa[i]) : zero16)
#define LDB_(S, i) S##b##i = *((kok && okb[i]) ? reinterpret_cast<const uint4*>(pb[i]) : zero16)
  // loads one stage into register set S; `valid` false (past the last stage) turns every load into a
  // read of the zero word, so the steady-state loop needs no branch around its loads
#define FETCH(S, valid)                                                                                   \
  do {                                                                                                    \
    const bool kok = (valid) && (k0 + ckc < Kseg);                                                        \
    LDA_(S, 0); LDA_(S, 1); LDA_(S, 2); LDA_(S, 3); LDB_(S, 0); LDB_(S, 1);                               \
  } while (0)
#define STA_(S, i) *reinterpret_cast<uint4*>(sa_ + (crow + i * 64) * ROWB + ckc * 2) = S##a##i
#define STB_(S, i) *reinterpret_cast<uint4*>(sb_ + (crow + i * 64) * ROWB + ckc * 2) = S##b##i
#define STASH(S, buf_)                                                                                    \
  do {                                                                                                    \
    char* sa_ = smem + (buf_) * STAGE;                                                                    \
    char* sb_ = sa_ + A_STAGE;                                                                            \
    STA_(S, 0); STA_(S, 1); STA_(S, 2); STA_(S, 3); STB_(S, 0); STB_(S, 1);                               \
  } while (0)
#define ADVANCE()                                                                                         \
  do {                                                                                                    \
    k0 += BK;                                                                                             \
    _Pragma("unroll") for (int i = 0; i < A_CH; ++i) pa[i] += BK;                                         \
    _Pragma("unroll") for (int i = 0; i < B_CH; ++i) pb[i] += BK;                                         \
    if (k0 >= kend) {                                                                                     \
      bool f_;                                                                                            \
      OPEN_SEG(f_);                                                                                       \
      (void)f_;                                                                                           \
    }                                                                                                     \
  } while (0)
#define COMPUTE(buf_)                                                                                     \
  do {                                                                                                    \
    const char* sa_ = smem + (buf_) * STAGE + (wm * 64 + (lane & 31)) * ROWB + (lane >> 5) * 16;         \
    const char* sb_ = smem + (buf_) * STAGE + A_STAGE + (wn * 64 + (lane & 31)) * ROWB + (lane >> 5) * 16; \
    _Pragma("unroll") for (int sub = 0; sub < BK / 16; ++sub) {                                           \
      uint4 fa[2], fb[2];                                                                                 \
      _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                       \
          fa[i] = *reinterpret_cast<const uint4*>(sa_ + i * 32 * ROWB + sub * 32);                        \
      _Pragma("unroll") for (int j = 0; j < 2; ++j)                                                       \
          fb[j] = *reinterpret_cast<const uint4*>(sb_ + j * 32 * ROWB + sub * 32);                        \
      _Pragma("unroll") for (int i = 0; i < 2; ++i) _Pragma("unroll") for (int j = 0; j < 2; ++j)         \
          acc[i][j] = HALF ? __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fa[i]),     \
                                                                    __builtin_bit_cast(f16x8, fb[j]), acc[i][j], 0, 0, 0)  \
                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),   \
                                                                     __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0); \
    }                                                                                                     \
  } while (0)
  // Global loads may not be scheduled across this point (the scheduler otherwise sinks them below
  // the MFMA block and exposes their latency); ALU, MFMA and LDS instructions may.
#define PIN_VMEM() __builtin_amdgcn_sched_barrier(0x1 | 0x2 | 0x4 | 0x8 | 0x80 | 0x100 | 0x200)

  // number of K stages over all segments
  int n_stage = 0;
  for (int sgi = 0; sgi < a.nseg; ++sgi) {
    int kb, ke;
    seg_range(a, sgi, m0, &kb, &ke);
    if (ke > kb) n_stage += (ke - kb + BK - 1) / BK;
  }
  const bool probe = a.clk != nullptr && blockIdx.x == 0 && blockIdx.z == 0;
  long long c_start = 0, w_start = 0;
  if (probe) c_start = clock64(), w_start = wall_clock64();
  if (n_stage > 0) {
    bool f0;
    OPEN_SEG(f0);
    (void)f0;
    FETCH(r, true);  // stage 0
    ADVANCE();
    FETCH(q, n_stage > 1);  // stage 1
    ADVANCE();
    STASH(r, 0);
    __syncthreads();
    // Straight-line body over PAIRS of stages (no exit in the middle: with one the compiler kept two
    // copies of the accumulators and shuffled them between register files).  At the top LDS buffer 0
    // holds stage st, set q holds stage st+1 (in flight), the cursor points at stage st+2.  With an
    // odd number of stages the last half-iteration multiplies a stage of zeros.
    for (int st = 0; st < n_stage; st += 2) {
      FETCH(r, st + 2 < n_stage);
      ADVANCE();
      PIN_VMEM();
      COMPUTE(0);
      STASH(q, 1);  // stage st+1 (zeros past the end)
      __syncthreads();
      FETCH(q, st + 3 < n_stage);
      ADVANCE();
      PIN_VMEM();
      COMPUTE(1);
      STASH(r, 0);  // stage st+2
      __syncthreads();
    }
  }
  if (probe && tid == 0) a.clk[0] = clock64() - c_start, a.clk[1] = wall_clock64() - w_start;
#undef OPEN_SEG
#undef FETCH
#undef LDA_
#undef LDB_
#undef STA_
#undef STB_
#undef STASH
#undef ADVANCE
#undef COMPUTE
#undef PIN_VMEM

  // ---- epilogue: lane holds rows 8*(v/4) + 4*(lane/32) + v%4 of column lane%32 of each 32x32 tile ----
  const int col_l = lane & 31, rgrp = (lane >> 5) * 4;
  unsigned short* Cb = a.Cb ? a.Cb + z0 * a.cb_bs0 + z1 * a.cb_bs1 + z2 * a.cb_bs2 : nullptr;
  float* Cf = a.Cf ? a.Cf + z0 * a.cf_bs0 + z1 * a.cf_bs1 + z2 * a.cf_bs2 : nullptr;
  const float* Rs = a.res ? a.res + z0 * a.cf_bs0 + z1 * a.cf_bs1 + z2 * a.cf_bs2 : nullptr;
  unsigned short* Ct = a.Ct ? a.Ct + z0 * a.ct_bs0 + z1 * a.ct_bs1 + z2 * a.ct_bs2 : nullptr;
  // Row-major outputs go through LDS (free after the K loop's last barrier; each wave uses a region of its own) so
  // that every global access is 16 bytes per lane along a row: 64-column rows of fp32 are 256 contiguous bytes,
  // the residual is read the same way, and all residual loads of a 32-row slab are in flight together.
  constexpr int ER = 72 * 4;  // staged row: 64 fp32 + 8 pad (4 rows further = 32 banks further)
  static_assert(8 * 32 * ER <= LDS_BYTES, "epilogue staging must fit the K-loop buffers");
  char* ebuf = smem + wave * (32 * ER);
  const bool vok = ((a.ldcf | a.ldcb) & 3) == 0 && ((reinterpret_cast<uintptr_t>(Cf) | reinterpret_cast<uintptr_t>(Rs)) & 15) == 0 &&
                   (reinterpret_cast<uintptr_t>(Cb) & 7) == 0;
  // whole rows of eight 16-bit columns: N and the row stride multiples of 8, 16-byte aligned base
  const bool vok8 = ((a.ldcb | a.N) & 7) == 0 && (reinterpret_cast<uintptr_t>(Cb) & 15) == 0;
  if (Cf || Cb || EPI != GEMM_EPI_NONE) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          *reinterpret_cast<float*>(ebuf + (8 * (v >> 2) + rgrp + (v & 3)) * ER + (j * 32 + col_l) * 4) = acc[i][j][v] * a.alpha;
      __builtin_amdgcn_wave_barrier();
      if (EPI != GEMM_EPI_NONE || (!Cf && vok8)) {  // 16-bit outputs only: eight columns (16 bytes) per lane, eight rows per pass
        const int c8 = (lane & 7) * 8, n8 = n0 + wn * 64 + c8;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int row = it * 8 + (lane >> 3);
          const int m = m0 + wm * 64 + i * 32 + row;
          const float4 lo = *reinterpret_cast<const float4*>(ebuf + row * ER + c8 * 4);
          const float4 hi = *reinterpret_cast<const float4*>(ebuf + row * ER + c8 * 4 + 16);
          if (m >= a.M || n8 >= a.N) continue;
          float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          auto pack = [](const float* v) {
            return HALF ? make_uint4(pack_h2(v[0], v[1]), pack_h2(v[2], v[3]), pack_h2(v[4], v[5]), pack_h2(v[6], v[7]))
                        : make_uint4(pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7]));
          };
          auto unpack = [](const uint4& w, float* v) {
            if (HALF) unpack8h(w, v);
            else unpack8(w, v);
          };
          if (EPI == GEMM_EPI_SILU_MUL) {
            float av[8], uv[8], mv[8];
            unpack(*reinterpret_cast<const uint4*>(a.e0 + (long long)m * a.lde + n8), av);
            const uint4 up = pack(x);
            unpack(up, uv);  // the rounded u, as the backward pass will read it
#pragma unroll
            for (int e = 0; e < 8; ++e) mv[e] = av[e] / (1.f + __expf(-av[e])) * uv[e];
            *reinterpret_cast<uint4*>(Cb + (long long)m * a.ldcb + n8) = up;
            *reinterpret_cast<uint4*>(a.o0 + (long long)m * a.lde + n8) = pack(mv);
          } else if (EPI == GEMM_EPI_SWIGLU_BWD) {
            float av[8], uv[8], oa[8], ou[8];
            unpack(*reinterpret_cast<const uint4*>(a.e0 + (long long)m * a.lde + n8), av);
            unpack(*reinterpret_cast<const uint4*>(a.e1 + (long long)m * a.lde + n8), uv);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float sg = 1.f / (1.f + __expf(-av[e]));
              oa[e] = x[e] * uv[e] * sg * (1.f + av[e] * (1.f - sg));
              ou[e] = x[e] * av[e] * sg;
            }
            *reinterpret_cast<uint4*>(a.o0 + (long long)m * a.lde + n8) = pack(oa);
            *reinterpret_cast<uint4*>(a.o1 + (long long)m * a.lde + n8) = pack(ou);
          } else {
            *reinterpret_cast<uint4*>(Cb + (long long)m * a.ldcb + n8) = pack(x);
          }
        }
        __builtin_amdgcn_wave_barrier();
        continue;
      }
      const int c4 = (lane & 15) * 4, n = n0 + wn * 64 + c4;
      const bool nvec = vok && n + 3 < a.N;
      float4 rv[8];
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int m = m0 + wm * 64 + i * 32 + it * 4 + (lane >> 4);
        rv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (Rs && nvec && m < a.M) rv[it] = *reinterpret_cast<const float4*>(Rs + (long long)m * a.ldcf + n);
      }
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int row = it * 4 + (lane >> 4);
        const int m = m0 + wm * 64 + i * 32 + row;
        float4 o = *reinterpret_cast<const float4*>(ebuf + row * ER + c4 * 4);
        if (m >= a.M || n >= a.N) continue;
        if (nvec) {
          o.x += rv[it].x, o.y += rv[it].y, o.z += rv[it].z, o.w += rv[it].w;
          if (Cf) *reinterpret_cast<float4*>(Cf + (long long)m * a.ldcf + n) = o;
          if (Cb)
            *reinterpret_cast<uint2*>(Cb + (long long)m * a.ldcb + n) =
                HALF ? make_uint2(pack_h2(o.x, o.y), pack_h2(o.z, o.w)) : make_uint2(pack_bf2(o.x, o.y), pack_bf2(o.z, o.w));
        } else {
          const float ov[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < a.N) {
              float x = ov[e];
              if (Cf) {
                if (Rs) x += Rs[(long long)m * a.ldcf + n + e];
                Cf[(long long)m * a.ldcf + n + e] = x;
              }
              if (Cb) Cb[(long long)m * a.ldcb + n + e] = HALF ? f2h(x) : f2bf(x);
            }
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  // transposed 16-bit output straight from the accumulators (a lane holds runs of four rows of one column)
  if (Ct) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + col_l;
        if (n >= a.N) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int mb = m0 + wm * 64 + i * 32 + q * 8 + rgrp;
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[e] = acc[i][j][q * 4 + e] * a.alpha;
            if (Cf && Rs && mb + e < a.M) o[e] += Rs[(long long)(mb + e) * a.ldcf + n];
          }
          unsigned short* p = Ct + (long long)n * a.ldct + mb;
          if (mb + 3 < a.M && ((a.ldct & 3) == 0) && (reinterpret_cast<uintptr_t>(Ct) & 7) == 0) {
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

// ---- optional per-launch timing (harli_prof_*): two events around every n-th GEMM launch ----
namespace {
struct ProfRec {
  hipEvent_t e0, e1;
  double flops;
};
int g_prof_every = 0;       // 0: off; n: the launches whose running number is a multiple of n are timed
long long g_prof_seen = 0;  // launches since enabling
std::vector<ProfRec> g_prof;
}  // namespace

void gemm_prof_enable(int every) {
  g_prof_every = every > 0 ? every : 0;
  g_prof_seen = 0;
}

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

hipError_t GemmTimer::begin(double flops_of_launch, hipStream_t st) {
  if (!(g_prof_every > 0 && (g_prof_seen++ % g_prof_every) == 0)) return hipSuccess;
  hipEvent_t a, b;
  hipError_t e = hipEventCreate(&a);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&b);
  if (e != hipSuccess) return e;
  e0 = a, e1 = b, flops = flops_of_launch;
  return hipEventRecord(a, st);
}
hipError_t GemmTimer::end(hipStream_t st) {
  if (!e0) return hipSuccess;
  hipError_t e = hipEventRecord(static_cast<hipEvent_t>(e1), st);
  g_prof.push_back(ProfRec{static_cast<hipEvent_t>(e0), static_cast<hipEvent_t>(e1), flops});
  e0 = e1 = nullptr;
  return e;
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
  if (a.epi == GEMM_EPI_NONE && !a.Cb && !a.Cf && !a.Ct) return fail(HARLI_ERR_INVALID, "gemm: no output");
  if (a.epi != GEMM_EPI_NONE) {
    const bool silu = a.epi == GEMM_EPI_SILU_MUL;
    if ((a.epi != GEMM_EPI_SILU_MUL && a.epi != GEMM_EPI_SWIGLU_BWD) || batches != 1 || a.Cf || a.Ct || a.res || (a.N & 7) || (a.lde & 7) ||
        !a.e0 || !a.o0 || (silu ? (!a.Cb || (a.ldcb & 7) || ((uintptr_t)a.Cb & 15)) : (!a.e1 || !a.o1 || a.Cb)) ||
        (((uintptr_t)a.e0 | (uintptr_t)a.e1 | (uintptr_t)a.o0 | (uintptr_t)a.o1) & 15))
      return fail(HARLI_ERR_INVALID, "gemm: fused SwiGLU epilogue %d needs N, lde %% 8 == 0, aligned operands and its own outputs only", a.epi);
  }
  if (a.res && !a.Cf) return fail(HARLI_ERR_INVALID, "gemm: a residual needs the fp32 output");
  static bool attr_set = false;
  static uint4* zero16 = nullptr;  // 256 zero bytes in device memory, kept for the life of the process
  if (!attr_set) {
    HARLI_HIP(hipMalloc(reinterpret_cast<void**>(&zero16), 256));
    HARLI_HIP(hipMemset(zero16, 0, 256));
#define HARLI_GEMM_ATTR(H_, E_) \
  HARLI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<H_, E_>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES))
    HARLI_GEMM_ATTR(true, GEMM_EPI_NONE); HARLI_GEMM_ATTR(true, GEMM_EPI_SILU_MUL); HARLI_GEMM_ATTR(true, GEMM_EPI_SWIGLU_BWD);
    HARLI_GEMM_ATTR(false, GEMM_EPI_NONE); HARLI_GEMM_ATTR(false, GEMM_EPI_SILU_MUL); HARLI_GEMM_ATTR(false, GEMM_EPI_SWIGLU_BWD);
#undef HARLI_GEMM_ATTR
    attr_set = true;
  }
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  // slots: whole GM x GN blocks (tiles past the edge of the matrix return at once)
  const int GM = std::min(kGM, tiles_m), GN = std::min(kGN, tiles_n);
  const int total = ((tiles_m + GM - 1) / GM) * ((tiles_n + GN - 1) / GN) * GM * GN, chunk = (total + 7) / 8;
  ProfRec rec{};
  const bool timed = g_prof_every > 0 && (g_prof_seen++ % g_prof_every) == 0;
  if (timed) {
    HARLI_HIP(hipEventCreate(&rec.e0));
    HARLI_HIP(hipEventCreate(&rec.e1));
    rec.flops = gemm_flops(a, batches);
    HARLI_HIP(hipEventRecord(rec.e0, st));
  }
#define HARLI_GEMM_LAUNCH(H_, E_) \
  hipLaunchKernelGGL((k_gemm<H_, E_>), dim3(chunk * 8, 1, batches), dim3(NT), LDS_BYTES, st, a, tiles_n, total, chunk, GM, GN, zero16)
  if (a.half) {
    if (a.epi == GEMM_EPI_SILU_MUL) HARLI_GEMM_LAUNCH(true, GEMM_EPI_SILU_MUL);
    else if (a.epi == GEMM_EPI_SWIGLU_BWD) HARLI_GEMM_LAUNCH(true, GEMM_EPI_SWIGLU_BWD);
    else HARLI_GEMM_LAUNCH(true, GEMM_EPI_NONE);
  } else {
    if (a.epi == GEMM_EPI_SILU_MUL) HARLI_GEMM_LAUNCH(false, GEMM_EPI_SILU_MUL);
    else if (a.epi == GEMM_EPI_SWIGLU_BWD) HARLI_GEMM_LAUNCH(false, GEMM_EPI_SWIGLU_BWD);
    else HARLI_GEMM_LAUNCH(false, GEMM_EPI_NONE);
  }
#undef HARLI_GEMM_LAUNCH
  if (timed) {
    HARLI_HIP(hipEventRecord(rec.e1, st));
    g_prof.push_back(rec);
  }
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}

}  // namespace harli
